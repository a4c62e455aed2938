"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs, element by element (see parity_util for the tolerances)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2604_04736_amd import workloads as W

import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hot():
    from paper_2604_04736_amd import binding
    binding.lib()          # a missing library is an error, never a skip
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


DEV = "cuda:0"


def _say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ whole small configs

@pytest.mark.parametrize("name", ["C1", "C2"])
def test_config_full_elementwise(oracle, hot, name):
    wl = W.CONFIGS[name]
    _say("case", name, wl)
    x = W.make_inputs(wl, DEV)
    rep = P.check_all(oracle, hot, x, wl)
    _say(name, rep)


# ------------------------------------------------------------------ scaled C3 / C5, launch shapes

LAUNCHES = [dict(), dict(chunks=1, unroll=1), dict(chunks=1, unroll=4, nontemporal=1),
            dict(chunks=2, unroll=2, nontemporal=1), dict(chunks=4, unroll=4, nontemporal=1),
            dict(chunks=4, unroll=1, grid_blocks=7), dict(chunks=2, unroll=4, grid_blocks=65536)]


@pytest.mark.parametrize("launch", LAUNCHES, ids=lambda d: "-".join(f"{k}{v}" for k, v in d.items()) or "default")
def test_scaled_c3_several_tiles_and_ragged_tail(oracle, hot, launch):
    # 16 samples, packed rows, N spans many tiles and ends 1 column past a multiple of 4
    wl = W.scaled(W.CONFIGS["C3"], 300_001)
    _say("case scaled C3", wl.n_weights, launch)
    x = W.make_inputs(wl, DEV)
    _say(P.check_all(oracle, hot, x, wl, launch=launch))


@pytest.mark.parametrize("offset", [0, 1, 3])
@pytest.mark.parametrize("launch", [dict(), dict(chunks=4, unroll=4, nontemporal=1), dict(chunks=1, unroll=2)],
                         ids=["default", "c4u4nt", "c1u2"])
def test_scaled_c5_adversarial_unaligned(oracle, hot, launch, offset):
    wl = W.scaled(W.CONFIGS["C5"], 400_003)
    _say("case scaled C5", wl.n_weights, launch, "offset", offset)
    x = W.make_inputs(wl, DEV, base_offset=offset)
    assert x["eps"].data_ptr() % 16 == 4 * offset
    _say(P.check_all(oracle, hot, x, wl, launch=launch))


# ------------------------------------------------------------------ edge sizes

def _random_case(n, ld, s, seed, dev=DEV):
    g = torch.Generator().manual_seed(seed)
    mu = torch.randn(n, generator=g)
    sigma = torch.exp(torch.randn(n, generator=g) * 2.0)
    eps = torch.full((s, ld), float("nan"))
    G = torch.full((s, ld), float("nan"))
    eps[:, :n] = torch.randn(s, n, generator=g)
    G[:, :n] = torch.randn(s, n, generator=g) * 3.0
    return {k: v.to(dev) for k, v in dict(mu=mu, sigma=sigma, eps=eps, G=G).items()}


class _WL:
    def __init__(self, n, ld, s_local, s_total, dsize):
        self.n_weights, self.ld, self.s_local, self.s_total, self.dataset_size = n, ld, s_local, s_total, dsize


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 7, 255, 1023, 1024, 1025, 2047, 2048, 2051, 4097, 8191])
def test_edge_sizes_packed_and_padded(oracle, hot, n):
    for s, s_total in [(1, 1), (3, 7), (5, 5), (17, 34)]:
        for ld in sorted({n, n + 1, hot.hot_recommended_ld(n)}):
            _say("case edge n", n, "ld", ld, "s", s)
            x = _random_case(n, ld, s, seed=n * 131 + s)
            wl = _WL(n, ld, s, s_total, 321.0)
            P.check_all(oracle, hot, x, wl)
            P.check_all(oracle, hot, x, wl, launch=dict(chunks=1, unroll=1, grid_blocks=1), flags=hot.HOT_REDUCE_MEAN)
            P.check_all(oracle, hot, x, wl, launch=dict(chunks=2, unroll=2), flags=hot.HOT_REDUCE_NONE)


def test_mean_convention_and_sharding_over_plans(oracle, hot):
    # Algorithm 2 on P groups of samples summed equals Algorithm 1 on all samples
    n, s, dsize = 70_001, 16, 45000.0
    x = _random_case(n, n, s, seed=5)
    wl = _WL(n, n, s, s, dsize)
    _, _, gmu_all, gsig_all = P.run_hip(hot, x, n, n, s, s, dsize)
    h = P.host(x)
    P.check_grads(oracle, h, gmu_all.cpu().numpy(), gsig_all.cpu().numpy(), n, s, dsize)
    for parts in (2, 4, 8, 16):
        per = s // parts
        acc_mu = torch.zeros(n, dtype=torch.float64, device=DEV)
        acc_sg = torch.zeros(n, dtype=torch.float64, device=DEV)
        avg_mu = torch.zeros_like(acc_mu)
        avg_sg = torch.zeros_like(acc_sg)
        for p in range(parts):
            xp = dict(mu=x["mu"], sigma=x["sigma"], eps=x["eps"][p * per:(p + 1) * per],
                      G=x["G"][p * per:(p + 1) * per])
            _, _, a, b = P.run_hip(hot, xp, n, n, per, s, dsize)
            acc_mu += a.double()
            acc_sg += b.double()
            _, _, a, b = P.run_hip(hot, xp, n, n, per, s, dsize, flags=hot.HOT_REDUCE_MEAN)
            avg_mu += a.double() / parts
            avg_sg += b.double() / parts
        # each part was rounded to fp32 once: compare the recombined result with the oracle
        # under a tolerance widened by the number of parts
        for got_mu, got_sg in ((acc_mu, acc_sg), (avg_mu, avg_sg)):
            gm64, gs64 = oracle.grad(h["mu"], h["sigma"], h["eps"], h["G"], s, dsize)
            g, k = P.gk(s, s, dsize)
            G64 = h["G"].astype(np.float64)
            e64 = h["eps"].astype(np.float64)
            tol_mu = P.RTOL * (g * np.abs(G64).sum(0) + k * np.abs(h["mu"]))
            tol_sg = P.RTOL * (g * np.abs(G64 * e64).sum(0) + k * (h["sigma"] + 1.0 / h["sigma"]))
            assert np.all(np.abs(got_mu.cpu().numpy() - gm64) <= tol_mu)
            assert np.all(np.abs(got_sg.cpu().numpy() - gs64) <= tol_sg)


def test_kl_optional_and_outputs_independent_of_it(hot):
    n, s = 10_000, 3
    x = _random_case(n, n, s, seed=9)
    w1, kl1, _, _ = P.run_hip(hot, x, n, n, s, s, 10.0, want_kl=True)
    w2, kl2, _, _ = P.run_hip(hot, x, n, n, s, s, 10.0, want_kl=False)
    assert kl2 is None and torch.equal(w1, w2) and kl1.item() > 0


def test_bitwise_determinism_over_repeated_launches(hot):
    wl = W.scaled(W.CONFIGS["C3"], 1_000_003)
    x = W.make_inputs(wl, DEV)
    n = wl.n_weights
    plan = hot.hot_create(n, wl.ld, wl.s_local, wl.s_total, wl.dataset_size, 0)
    outs = []
    for rep in range(4):
        w = torch.empty_like(x["eps"])
        kl = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
        gmu, gsig = torch.empty_like(x["mu"]), torch.empty_like(x["mu"])
        hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
        hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], gmu, gsig)
        torch.cuda.synchronize()
        outs.append((w, kl, gmu, gsig))
    hot.hot_destroy(plan)
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert torch.equal(a, b)


@pytest.mark.parametrize("n,launch", [(64 * 4096, None), (64 * 4096 + 1, None), (63 * 4096 + 5, None), (1_000_003, {"grid_blocks": 8}),
                                      (1_000_003, {"grid_blocks": 64, "chunks": 1}), (300_000, {"grid_blocks": 65, "chunks": 1})])
def test_kl_on_either_side_of_the_small_grid_boundary(oracle, hot, n, launch):
    """Up to 64 workgroups the forward kernel adds its KL partials itself (the last workgroup to
    arrive does it); above, a second kernel does.  Both sides of the boundary, grids forced small
    on larger inputs, and repeated calls on one plan (the arrival counter must be back at zero)."""
    print("case small-grid KL", n, launch, flush=True)
    x = _random_case(n, n, 2, seed=n % 1000)
    h = P.host(x)
    plan = hot.hot_create(n, n, 2, 2, 100.0, 0)
    if launch:
        hot.hot_set_launch(plan, hot.HOT_KERNEL_FORWARD, **launch)
        hot.hot_set_launch(plan, hot.HOT_KERNEL_FORWARD_RNG, **launch)
    w = torch.empty_like(x["eps"])
    kls = []
    for rep in range(5):
        kl = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
        if rep == 3:
            hot.hot_forward_rng(plan, hot.hot_rng(seed=5, step=rep, first_sample=0), x["mu"], x["sigma"], w, kl)
        else:
            hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
        torch.cuda.synchronize()
        kls.append(kl.item())
    hot.hot_destroy(plan)
    P.check_kl(oracle, h, kls[0])
    assert all(k == kls[0] for k in kls), kls


@pytest.mark.parametrize("n,offset", [(1, 0), (5, 1), (4097, 0), (262_144, 0), (300_001, 3), (5_000_003, 0)])
def test_kl_alone_equals_the_forward_call(oracle, hot, n, offset):
    """hot_kl against the oracle and, bit for bit, against the KL that hot_forward returns."""
    print("case kl alone", n, offset, flush=True)
    x = _random_case(n, n, 2, seed=n % 997)
    if offset:
        buf = {k: torch.empty(v.numel() + offset, device=DEV) for k, v in x.items()}
        for k in x:
            buf[k][offset:].view(x[k].shape).copy_(x[k])
        x = {k: buf[k][offset:].view(x[k].shape) for k in x}
    plan = hot.hot_create(n, n, 2, 2, 10.0, 0)
    kl_f = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    kl_a = torch.full((1,), -2.0, dtype=torch.float64, device=DEV)
    hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], torch.empty_like(x["eps"]), kl_f)
    hot.hot_kl(plan, x["mu"], x["sigma"], kl_a)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    assert kl_a.item() == kl_f.item()
    P.check_kl(oracle, P.host(x), kl_a.item())


def test_ieee_propagation_for_sigma_outside_the_domain(oracle, hot):
    n, s = 2051, 2
    x = _random_case(n, n, s, seed=11)
    x["sigma"][17] = 0.0
    w, kl, gmu, gsig = P.run_hip(hot, x, n, n, s, s, 10.0)
    assert kl.item() == float("inf") and gsig[17].item() == float("-inf")
    assert torch.isfinite(gmu).all() and torch.isfinite(w).all()
    assert torch.isfinite(gsig).sum().item() == n - 1
    h = P.host(x)
    assert oracle.kl(h["mu"], h["sigma"]) == float("inf")
    x["sigma"][17] = -1.0
    _, kl, _, _ = P.run_hip(hot, x, n, n, s, s, 10.0)
    assert np.isnan(kl.item()) and np.isnan(oracle.kl(P.host(x)["mu"], P.host(x)["sigma"]))


def test_cancellation_in_w_is_correctly_rounded(oracle, hot):
    # mu = -sigma*eps up to one rounding: a separate multiply and add would lose all digits
    n, s = 4099, 2
    g = torch.Generator().manual_seed(3)
    sigma = torch.rand(n, generator=g) + 0.5
    eps = torch.randn(s, n, generator=g)
    mu = -(sigma * eps[0])
    x = {k: v.to(DEV) for k, v in dict(mu=mu, sigma=sigma, eps=eps, G=torch.ones(s, n)).items()}
    w, _, _, _ = P.run_hip(hot, x, n, n, s, s, 10.0)
    P.check_w(oracle, P.host(x), w.cpu().numpy(), n)


def test_errors_from_the_c_abi(hot):
    L = hot.lib()
    with pytest.raises(hot.HotError):
        hot.hot_create(8, 8, 1, 1, 1.0, device=99)
    plan = hot.hot_create(1024, 1024, 2, 2, 1.0, 0)
    t = torch.zeros(4096, device=DEV)
    p = ctypes.c_void_p(t.data_ptr())
    odd = ctypes.c_void_p(t.data_ptr() + 2)
    assert L.hot_forward(plan.handle, None, p, p, p, None, None) == hot.HOT_EINVAL
    assert L.hot_forward(plan.handle, odd, p, p, p, None, None) == hot.HOT_EINVAL
    assert L.hot_forward(plan.handle, p, p, p, p, ctypes.c_void_p(t.data_ptr() + 4), None) == hot.HOT_EINVAL
    assert L.hot_backward(plan.handle, p, p, p, p, p, None, None) == hot.HOT_EINVAL
    assert L.hot_backward(plan.handle, p, p, p, p, p, odd, None) == hot.HOT_EINVAL
    with pytest.raises(hot.HotError):
        hot.hot_set_launch(plan, hot.HOT_KERNEL_FORWARD, chunks=3)
    with pytest.raises(hot.HotError):
        hot.hot_set_launch(plan, 5, chunks=2)
    with pytest.raises(hot.HotError):
        hot.hot_set_launch(plan, hot.HOT_KERNEL_FORWARD, grid_blocks=1 << 20)
    with pytest.raises(ValueError):
        hot.hot_forward(plan, t[:1000], t[:1024], t.view(2, 2048)[:, :1024], t.view(2, 2048)[:, :1024])
    with pytest.raises(TypeError):
        hot.hot_forward(plan, t[:1024].cpu(), t[:1024], t[:2048].view(2, 1024), t[:2048].view(2, 1024))
    cfg = hot.hot_get_launch(plan, hot.HOT_KERNEL_BACKWARD)
    # two samples, few weights: one chunk per thread, both rows in flight; non-temporal hints at every size
    assert cfg["unroll"] == 2 and cfg["nontemporal"] == 1 and cfg["chunks"] == 1 and cfg["grid_blocks"] > 0
    assert hot.hot_get_launch(plan, hot.HOT_KERNEL_FORWARD)["chunks"] == 1
    hot.hot_destroy(plan)
    big = hot.hot_create(1 << 26, 1 << 26, 2, 2, 1.0, 0)      # 512 MiB of samples: four chunks, non-temporal
    cfg = hot.hot_get_launch(big, hot.HOT_KERNEL_BACKWARD)
    assert cfg["chunks"] == 4 and cfg["nontemporal"] == 1
    hot.hot_destroy(big)
    many = hot.hot_create(1 << 22, 1 << 22, 16, 16, 1.0, 0)
    assert hot.hot_get_launch(many, hot.HOT_KERNEL_FORWARD_RNG)["chunks"] == 1
    assert hot.hot_get_launch(many, hot.HOT_KERNEL_BACKWARD)["chunks"] == 4
    hot.hot_destroy(many)
    # chunks per thread follow the number of column tiles: 2.7 M weights are 658 tiles of 4096 (2.6 rounds of the
    # 256 compute units) -> smaller tiles; 1 M weights are 256 tiles of 4096 -> 512 tiles of 2048
    for n_w, want in ((2_693_578, 1), (1 << 20, 2), (6_291_456, 4), (7_700_003, 4), (300_000, 1)):
        pl = hot.hot_create(n_w, n_w, 4, 16, 1.0, 0)
        assert hot.hot_get_launch(pl, hot.HOT_KERNEL_FORWARD)["chunks"] == want, n_w
        hot.hot_destroy(pl)
    hot.hot_destroy(plan)      # second destroy of the wrapper is a no-op


def test_probe_copy_is_exact(hot):
    for count in (4, 1024, 4096 + 4, 1_000_004):
        src = torch.randn(count, device=DEV)
        for nt in range(2):
            dst = torch.zeros(count + 8, device=DEV)
            hot.hot_probe_copy(dst[4:4 + count], src, nt)
            torch.cuda.synchronize()
            assert torch.equal(dst[4:4 + count], src)
            assert dst[:4].abs().sum().item() == 0 and dst[4 + count:].abs().sum().item() == 0
    with pytest.raises(hot.HotError):
        hot.lib()   # keep the handle alive
        hot.hot_probe_copy(torch.zeros(6, device=DEV)[1:5], torch.zeros(4, device=DEV))


def test_probe_streams_sums_its_read_streams(hot):
    count = 100_000                      # floats per stream, a multiple of 4
    for reads, writes in [(1, 0), (1, 1), (2, 2), (4, 2), (6, 2), (6, 0), (3, 1), (5, 2), (7, 1), (18, 16), (34, 2), (15, 13),
                          (28, 2), (64, 64), (3, 3)]:
        arena = torch.randn((reads + writes) * count, device=DEV)
        before = arena.clone()
        hot.hot_probe_streams(arena, 4 * count, reads, writes)
        torch.cuda.synchronize()
        assert torch.equal(arena[:reads * count], before[:reads * count])
        if reads > 6 or writes > 2:        # the looping kernel adds four streams at a time onto a running sum from zero
            want = torch.zeros(count, device=DEV)
            for r0 in range(0, reads - reads % 4, 4):
                for r in range(r0, r0 + 4):
                    want += before[r * count:(r + 1) * count]
            for r in range(reads - reads % 4, reads):
                want += before[r * count:(r + 1) * count]
        else:
            want = before[:count].clone()
            for r in range(1, reads):
                want += before[r * count:(r + 1) * count]
        for w in range(writes):
            assert torch.equal(arena[(reads + w) * count:(reads + w + 1) * count], want)
    # streams off the 16-byte grid (a pitch of 4 * 100_003 bytes): whole quads of every stream summed, the last three
    # floats of every write stream and everything else left alone
    count = 100_003
    for reads, writes in [(2, 1), (15, 13), (5, 2)]:
        arena = torch.randn((reads + writes) * count + 8, device=DEV)
        before = arena.clone()
        hot.hot_probe_streams(arena, 4 * count, reads, writes)
        torch.cuda.synchronize()
        assert torch.equal(arena[:reads * count], before[:reads * count])
        want = torch.zeros(count - 3, device=DEV)
        for r0 in range(0, reads - reads % 4, 4):
            for r in range(r0, r0 + 4):
                want += before[r * count:(r + 1) * count - 3]
        for r in range(reads - reads % 4, reads):
            want += before[r * count:(r + 1) * count - 3]
        for w in range(writes):
            lo = (reads + w) * count
            assert torch.equal(arena[lo:lo + count - 3], want)
            assert torch.equal(arena[lo + count - 3:lo + count], before[lo + count - 3:lo + count])
        assert torch.equal(arena[(reads + writes) * count:], before[(reads + writes) * count:])
    with pytest.raises(hot.HotError):
        hot.hot_probe_streams(torch.zeros(1024, device=DEV), 16, 65, 1)
    with pytest.raises(hot.HotError):
        hot.hot_probe_streams(torch.zeros(1024, device=DEV), 18, 2, 1)
    with pytest.raises(hot.HotError):
        hot.hot_probe_streams(torch.zeros(1024, device=DEV), 20, 2, 0)
    with pytest.raises(hot.HotError):
        hot.hot_probe_streams(torch.zeros(64, device=DEV), 16, 7, 0)
    with pytest.raises(ValueError):
        hot.hot_probe_streams(torch.zeros(4, device=DEV), 16, 2, 2)


def test_runs_on_a_side_stream(oracle, hot):
    wl = W.scaled(W.CONFIGS["C2"], 100_000)
    x = W.make_inputs(wl, DEV)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        rep = P.check_all(oracle, hot, x, wl)
    _say(rep)


# ------------------------------------------------------------------ full sizes, bench launch shape

def _column_blocks(n, rng, count, width):
    blocks = [(0, min(width, n)), (max(0, n - width - 3), n)]
    for _ in range(count):
        a = int(rng.integers(0, max(1, n - width)))
        blocks.append((a, min(n, a + width)))
    return blocks


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_full_size_sampled_blocks_and_whole_kl(oracle, hot, name):
    """At the benchmark's sizes and default launch shape: the KL term over all weights, and
    w, grad_mu, grad_sigma on contiguous column blocks (first, last with the ragged tail, and
    random ones) that the oracle recomputes from the same bytes."""
    wl = W.CONFIGS[name]
    _say("case full", name, wl.n_weights, wl.s_local)
    x = W.make_inputs(wl, DEV)
    n, ld = wl.n_weights, wl.ld
    w, kl, gmu, gsig = P.run_hip(hot, x, n, ld, wl.s_local, wl.s_total, wl.dataset_size)
    _say("ran", name)
    h_mu, h_sigma = x["mu"].cpu().numpy(), x["sigma"].cpu().numpy()
    rel = P.check_kl(oracle, {"mu": h_mu, "sigma": h_sigma}, kl.item())
    _say("KL ok", kl.item(), rel)
    rng = np.random.default_rng(wl.seed)
    for a, b in _column_blocks(n, rng, 24, 40_000):
        h = {"mu": h_mu[a:b].copy(), "sigma": h_sigma[a:b].copy(),
             "eps": np.ascontiguousarray(x["eps"][:, a:b].cpu().numpy()),
             "G": np.ascontiguousarray(x["G"][:, a:b].cpu().numpy())}
        P.check_w(oracle, h, w[:, a:b].cpu().numpy(), b - a)
        P.check_grads(oracle, h, gmu[a:b].cpu().numpy(), gsig[a:b].cpu().numpy(), b - a,
                      wl.s_total, wl.dataset_size)
    # properties that hold at any size: every output written, finite, and w rows differ
    assert torch.isfinite(w).all() and torch.isfinite(gmu).all() and torch.isfinite(gsig).all()


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_full_size_every_element(oracle, hot, name):
    """Every element of w, grad_mu and grad_sigma and the whole KL term at the benchmark's sizes and default
    launch shape (C4, the workload the metric is quoted on, block by block to bound host memory)."""
    wl = W.CONFIGS[name]
    _say("case every element", name)
    x = W.make_inputs(wl, DEV)
    if wl.items > 200_000_000:
        _say(P.check_all_chunked(oracle, hot, x, wl, say=_say))
    else:
        _say(P.check_all(oracle, hot, x, wl))


def test_indices_beyond_32_bits(oracle, hot):
    """S_loc * ld = 4.8e9 elements: row offsets pass 2^32, and there are more column tiles than the
    grid bound, so workgroups stride over tiles.  Sampled windows in the last rows against the oracle."""
    n, s = 1_200_000_003, 4
    _say("case huge", n, s)
    g = torch.Generator(device=DEV).manual_seed(7)
    mu = torch.randn(n, device=DEV, generator=g)
    sigma = torch.rand(n, device=DEV, generator=g) * 0.5 + 0.01
    eps = torch.randn(s, n, device=DEV, generator=g)
    G = torch.randn(s, n, device=DEV, generator=g)
    w = torch.empty(s, n, device=DEV)
    gmu, gsig = torch.empty(n, device=DEV), torch.empty(n, device=DEV)
    kl = torch.zeros(1, dtype=torch.float64, device=DEV)
    plan = hot.hot_create(n, n, s, 16, 45000.0, 0)
    hot.hot_forward(plan, mu, sigma, eps, w, kl)
    hot.hot_backward(plan, mu, sigma, eps, G, gmu, gsig)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    _say("ran huge")
    rng = np.random.default_rng(1)
    width = 10_000
    for a in [0, n - width, 1_073_741_824 - 5000, 805_306_368 - 17] + [int(v) for v in rng.integers(0, n - width, size=4)]:
        b = a + width
        h = {"mu": mu[a:b].cpu().numpy(), "sigma": sigma[a:b].cpu().numpy(),
             "eps": np.ascontiguousarray(eps[:, a:b].cpu().numpy()), "G": np.ascontiguousarray(G[:, a:b].cpu().numpy())}
        P.check_w(oracle, h, w[:, a:b].cpu().numpy(), width)
        P.check_grads(oracle, h, gmu[a:b].cpu().numpy(), gsig[a:b].cpu().numpy(), width, 16, 45000.0)
    del eps, G, w
    # the KL term of all 1.2e9 weights against the oracle, which takes them in blocks of 2^26 (the term is
    # additive over any partition of the weights; the oracle's pins include that)
    want = scale = 0.0
    for c0 in range(0, n, 1 << 26):
        hb = {"mu": mu[c0:c0 + (1 << 26)].cpu().numpy(), "sigma": sigma[c0:c0 + (1 << 26)].cpu().numpy()}
        want += oracle.kl(hb["mu"], hb["sigma"])
        scale += P.kl_scale(hb)
    _say("KL", kl.item(), "oracle", want, "difference over the sum of addend magnitudes", abs(kl.item() - want) / scale)
    assert abs(kl.item() - want) <= P.RTOL * scale
    assert abs(kl.item() - want) <= 1e-7 * abs(want)        # (far inside the tolerance: every addend is positive here)


def test_hip_graph_replays_equal_eager(hot):
    """The run calls neither allocate nor synchronise, so a stream capture takes them; every replay,
    with eager work in between, must reproduce the eager result bit for bit."""
    wl = W.CONFIGS["C1"]
    x = W.make_inputs(wl, DEV)
    plan = hot.hot_create(wl.n_weights, wl.ld, wl.s_local, wl.s_total, wl.dataset_size, 0)
    rngd = hot.hot_rng(seed=3, step=1, first_sample=0)

    def buffers():
        return (torch.zeros_like(x["eps"]), torch.zeros(1, dtype=torch.float64, device=DEV), torch.zeros_like(x["mu"]),
                torch.zeros_like(x["mu"]), torch.zeros_like(x["eps"]), torch.zeros_like(x["mu"]), torch.zeros_like(x["mu"]))

    def step(b):
        w, kl, gmu, gsig, w2, gmu2, gsig2 = b
        hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
        hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], gmu, gsig)
        hot.hot_forward_rng(plan, rngd, x["mu"], x["sigma"], w2, None)
        hot.hot_backward_rng(plan, rngd, x["mu"], x["sigma"], x["G"], gmu2, gsig2)

    eager = buffers()
    step(eager)
    torch.cuda.synchronize()
    captured = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(captured)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(captured)
    for rep in range(4):
        for t in captured:
            t.fill_(float(rep + 5)) if t.dtype == torch.float32 else t.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, captured):
            if a.dim() == 2:                # padding columns are never written: compare the payload
                a, b = a[:, :wl.n_weights], b[:, :wl.n_weights]
            assert torch.equal(a, b), rep
        scratch = torch.randn(1000, device=DEV).sum().item()      # eager work between replays
        assert scratch == scratch
    hot.hot_destroy(plan)


def test_random_shapes_offsets_and_launch_shapes(oracle, hot):
    """Seeded random draw of sizes, pitches, base offsets, sample counts and launch shapes, array and
    in-kernel eps paths, every output compared element by element."""
    rs = np.random.default_rng(2026)
    for case in range(40):
        n = int(rs.choice([rs.integers(1, 64), rs.integers(64, 5000), rs.integers(5000, 200_000)]))
        ld = int(n + rs.choice([0, 0, 1, 3, 4, 61]))
        s = int(rs.integers(1, 20))
        s_total = int(s * rs.integers(1, 5))
        offset = int(rs.choice([0, 0, 1, 2, 3]))
        launch = dict(chunks=int(rs.choice([1, 2, 4])), unroll=int(rs.choice([1, 2, 4])),
                      nontemporal=int(rs.integers(0, 2)), grid_blocks=int(rs.choice([0, 1, 3, 64])))
        flags = int(rs.integers(0, 3))        # sum, mean and unscaled reduce conventions
        _say("case random", case, n, ld, s, s_total, offset, launch, flags)
        g = torch.Generator().manual_seed(case)
        def place(t):
            buf = torch.empty(t.numel() + offset, device=DEV)
            v = buf[offset:].view(t.shape)
            v.copy_(t)
            return v
        pad = torch.full((s, ld - n), float("nan"))
        x = {"mu": place(torch.randn(n, generator=g)), "sigma": place(torch.exp(torch.randn(n, generator=g))),
             "eps": place(torch.cat([torch.randn(s, n, generator=g), pad], 1)),
             "G": place(torch.cat([torch.randn(s, n, generator=g) * 2, pad], 1))}
        wl = _WL(n, ld, s, s_total, 1234.5)
        P.check_all(oracle, hot, x, wl, launch=launch, flags=flags)
        # in-kernel eps: fused kernels against array kernels fed with the materialised draw
        rng = hot.hot_rng(seed=case * 7919 + 1, step=case, first_sample=case % 5)
        plan = hot.hot_create(n, ld, s, s_total, 1234.5, 0, flags)
        for kern in (hot.HOT_KERNEL_FORWARD_RNG, hot.HOT_KERNEL_BACKWARD_RNG):
            hot.hot_set_launch(plan, kern, **launch)
        eps = place(torch.zeros(s, ld))
        hot.hot_sample_eps(plan, rng, eps)
        w0, w1 = place(torch.zeros(s, ld)), place(torch.zeros(s, ld))
        o = [place(torch.zeros(n)) for _ in range(4)]
        hot.hot_forward(plan, x["mu"], x["sigma"], eps, w0, None)
        hot.hot_backward(plan, x["mu"], x["sigma"], eps, x["G"], o[0], o[1])
        hot.hot_forward_rng(plan, rng, x["mu"], x["sigma"], w1, None)
        hot.hot_backward_rng(plan, rng, x["mu"], x["sigma"], x["G"], o[2], o[3])
        torch.cuda.synchronize()
        hot.hot_destroy(plan)
        assert torch.equal(w0[:, :n], w1[:, :n]) and torch.equal(o[0], o[2]) and torch.equal(o[1], o[3])
        e64 = oracle.eps_normal(n, s, rng.seed, rng.step, rng.first_sample)
        assert np.abs(eps[:, :n].cpu().numpy() - e64).max() <= 2e-6 * 5.78


def test_rows_off_the_64_byte_grid(oracle, hot):
    """The forward kernel for rows of w that do not start on 64-byte boundaries (taken with non-temporal
    accesses: forced here, the default above 256 MiB): every base offset 0..15 floats of w, pitches of
    every residue class that matters, one to several rows, sizes around the 4096-column tile and the
    16-column halo, eps read (at its own, different alignment) and drawn, with and without KL, one
    workgroup striding over all windows and many.  Everything element by element against the oracle;
    the padding of w must stay untouched."""
    rs = np.random.default_rng(64)
    sizes = [1, 3, 15, 16, 17, 4095, 4096, 4097, 4096 + 15, 4096 + 16, 2 * 4096 - 1, 3 * 4096 + 5, 70_001]
    case = 0
    for n in sizes:
        for ld_pad in (0, 1, 4, 12, 16, 20):
            case += 1
            ld = n + ld_pad
            s = int(rs.integers(1, 6))
            w_off, e_off = int(rs.integers(0, 16)), int(rs.integers(0, 16))
            grid = int(rs.choice([0, 1, 3]))
            want_kl = bool(rs.integers(0, 2))
            _say("case off-grid", n, ld, s, w_off, e_off, grid, want_kl)
            g = torch.Generator().manual_seed(case)
            mu, sigma = torch.randn(n, generator=g), torch.exp(torch.randn(n, generator=g))
            eps_h = torch.cat([torch.randn(s, n, generator=g), torch.full((s, ld - n), float("nan"))], 1)

            def at(t, off, fill=None):
                buf = torch.full((t.numel() + 16,), 5.0 if fill is None else fill, device=DEV)
                v = buf[off:off + t.numel()].view(t.shape)
                if fill is None:
                    v.copy_(t)
                return v

            mu_d, sg_d, eps_d = at(mu, int(rs.integers(0, 4))), at(sigma, int(rs.integers(0, 4))), at(eps_h, e_off)
            plan = hot.hot_create(n, ld, s, 2 * s, 77.0, 0)
            for kern in (hot.HOT_KERNEL_FORWARD, hot.HOT_KERNEL_FORWARD_RNG):
                hot.hot_set_launch(plan, kern, nontemporal=1, grid_blocks=grid, chunks=4)
            # eps from its array
            w = at(eps_h, w_off, fill=123456.0)
            kl = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
            hot.hot_forward(plan, mu_d, sg_d, eps_d, w, kl if want_kl else None)
            torch.cuda.synchronize()
            h = {"mu": mu.numpy(), "sigma": sigma.numpy(), "eps": eps_h.numpy()}
            wh = w.cpu().numpy()
            assert np.all(wh[:, n:] == np.float32(123456.0)), "w padding was written"
            P.check_w(oracle, h, wh, n)
            if want_kl:
                P.check_kl(oracle, h, kl.item())
            else:
                assert kl.item() == -1.0
            # eps drawn in the kernel (always the general kernel) against the materialised draw fed to the
            # row-shifting kernel: the same w, bit for bit
            rng = hot.hot_rng(seed=case, step=3, first_sample=1)
            e_draw = at(eps_h, 4 * int(rs.integers(0, 4)), fill=0.0)
            hot.hot_sample_eps(plan, rng, e_draw)
            w0, w1 = at(eps_h, w_off, fill=123456.0), at(eps_h, w_off, fill=123456.0)
            kl0, kl1 = torch.zeros(1, dtype=torch.float64, device=DEV), torch.zeros(1, dtype=torch.float64, device=DEV)
            hot.hot_forward(plan, mu_d, sg_d, e_draw, w0, kl0)
            hot.hot_forward_rng(plan, rng, mu_d, sg_d, w1, kl1)
            torch.cuda.synchronize()
            assert torch.equal(w0, w1), "drawn and materialised eps give different w"
            assert abs(kl0.item() - kl1.item()) <= 1e-13 * P.kl_scale(h)
            hot.hot_destroy(plan)


def test_two_plans_on_two_streams_at_once(oracle, hot):
    wl = W.scaled(W.CONFIGS["C3"], 400_000)
    xa = W.make_inputs(wl, DEV)
    xb = {k: v.flip(-1).contiguous() for k, v in xa.items()}
    torch.cuda.synchronize()
    outs = []
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    plans = [hot.hot_create(wl.n_weights, wl.ld, wl.s_local, wl.s_total, wl.dataset_size, 0) for _ in range(2)]
    for rep in range(3):
        outs = []
        for st, plan, x in zip(streams, plans, (xa, xb)):
            with torch.cuda.stream(st):
                w = torch.empty_like(x["eps"])
                kl = torch.zeros(1, dtype=torch.float64, device=DEV)
                gmu, gsig = torch.empty_like(x["mu"]), torch.empty_like(x["mu"])
                hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
                hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], gmu, gsig)
                outs.append((w, kl, gmu, gsig))
        torch.cuda.synchronize()
    for plan in plans:
        hot.hot_destroy(plan)
    for x, (w, kl, gmu, gsig) in zip((xa, xb), outs):
        h = P.host(x)
        P.check_w(oracle, h, w.cpu().numpy(), wl.n_weights)
        P.check_kl(oracle, h, kl.item())
        P.check_grads(oracle, h, gmu.cpu().numpy(), gsig.cpu().numpy(), wl.n_weights, wl.s_total, wl.dataset_size)


def test_training_step_of_a_small_bayesian_mlp_matches_autograd(hot):
    """Algorithm 2 on one GPU around a real network: the library does the sample layer, torch autograd
    only the network; the resulting gradients of mu and sigma equal fp64 autograd of the whole objective."""
    torch.manual_seed(1)
    d_in, d_h, d_out, batch, s, dsize = 16, 32, 4, 64, 4, 45000.0
    n = d_in * d_h + d_h + d_h * d_out + d_out
    mu = (torch.randn(n) * 0.2).to(DEV)
    sigma = (torch.rand(n) * 0.1 + 0.02).to(DEV)
    xb = torch.randn(batch, d_in, device=DEV)
    yb = torch.randn(batch, d_out, device=DEV)
    rng = hot.hot_rng(seed=11, step=0, first_sample=0)

    def net_loss(w, x, y):
        o = 0
        w1 = w[o:o + d_in * d_h].view(d_h, d_in); o += d_in * d_h
        b1 = w[o:o + d_h]; o += d_h
        w2 = w[o:o + d_h * d_out].view(d_out, d_h); o += d_h * d_out
        b2 = w[o:o + d_out]
        return ((torch.tanh(x @ w1.T + b1) @ w2.T + b2 - y) ** 2).mean()

    plan = hot.hot_create(n, n, s, s, dsize, 0)
    w = torch.empty(s, n, device=DEV)
    kl = torch.zeros(1, dtype=torch.float64, device=DEV)
    hot.hot_forward_rng(plan, rng, mu, sigma, w, kl)
    G = torch.empty_like(w)
    for i in range(s):                       # the network's own forward / backward, per sample
        wi = w[i].clone().requires_grad_(True)
        net_loss(wi, xb, yb).backward()
        G[i] = wi.grad
    gmu, gsig = torch.empty(n, device=DEV), torch.empty(n, device=DEV)
    hot.hot_backward_rng(plan, rng, mu, sigma, G, gmu, gsig)
    eps = torch.empty(s, n, device=DEV)
    hot.hot_sample_eps(plan, rng, eps)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    # reference: the whole objective in fp64 on the CPU, differentiated by autograd
    m64 = mu.double().cpu().requires_grad_(True)
    s64 = sigma.double().cpu().requires_grad_(True)
    e64 = eps.double().cpu()
    data = sum(net_loss(m64 + s64 * e64[i], xb.double().cpu(), yb.double().cpu()) for i in range(s)) / s
    kl64 = 0.5 * (s64 ** 2 + m64 ** 2 - 1 - 2 * torch.log(s64)).sum()
    (data + kl64 / dsize).backward()
    assert abs(kl.item() - kl64.item()) <= 1e-7 * abs(kl64.item())
    Gh = G.double().cpu()
    tol_mu = 1e-4 * (Gh.abs().sum(0) / s + m64.detach().abs() / dsize)       # G itself is an fp32 autograd result
    tol_sg = 1e-4 * ((Gh * e64).abs().sum(0) / s + (s64.detach() + 1 / s64.detach()) / dsize)
    assert torch.all((gmu.double().cpu() - m64.grad).abs() <= tol_mu)
    assert torch.all((gsig.double().cpu() - s64.grad).abs() <= tol_sg)


@pytest.mark.parametrize("groups", [[1] * 6, [2, 4], [5, 1], [6]])
@pytest.mark.parametrize("use_rng", [False, True])
@pytest.mark.parametrize("n,ld,launch", [(50_003, 50_016, None), (70_001, 70_004, dict(chunks=4, unroll=4, nontemporal=1)),
                                         (70_001, 70_001, dict(chunks=4, unroll=2)), (9_000, 9_000, dict(chunks=2, unroll=1))],
                         ids=["default", "c4u4nt", "c4u2-unaligned", "c2u1"])
def test_backward_over_subsets_of_samples_accumulates_to_the_whole(oracle, hot, groups, use_rng, n, ld, launch):
    # (the launch shapes decide how the kernel fetches what it adds to: ahead of all stores through windows with
    # four rows in flight or drawn eps, chunk by chunk otherwise; full tiles and the narrow last one)
    s, s_total, dsize = 6, 12, 777.0
    x = _random_case(n, ld, s, seed=21)
    plan = hot.hot_create(n, ld, s, s_total, dsize, 0)
    if launch:
        for kern in (hot.HOT_KERNEL_BACKWARD, hot.HOT_KERNEL_BACKWARD_RNG):
            hot.hot_set_launch(plan, kern, **launch)
    rng = hot.hot_rng(seed=8, step=3, first_sample=6)
    if use_rng:
        hot.hot_sample_eps(plan, rng, x["eps"])
    whole_mu, whole_sg = torch.empty(n, device=DEV), torch.empty(n, device=DEV)
    if use_rng:
        hot.hot_backward_rng(plan, rng, x["mu"], x["sigma"], x["G"], whole_mu, whole_sg)
    else:
        hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], whole_mu, whole_sg)
    acc_mu = torch.full((n,), float("nan"), device=DEV)
    acc_sg = torch.full((n,), float("nan"), device=DEV)
    at = 0
    for i, g in enumerate(groups):
        hot.hot_backward_rows(plan, rng if use_rng else None, x["mu"], x["sigma"],
                              None if use_rng else x["eps"][at:at + g], x["G"][at:at + g], at,
                              accumulate=i > 0, add_kl=i == len(groups) - 1, grad_mu=acc_mu, grad_sigma=acc_sg)
        at += g
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    if len(groups) == 1:
        assert torch.equal(acc_mu, whole_mu) and torch.equal(acc_sg, whole_sg)
    h = P.host(x)
    # every partial call rounds the running sums to fp32 once: the usual tolerance covers it
    P.check_grads(oracle, h, acc_mu.cpu().numpy(), acc_sg.cpu().numpy(), n, s_total, dsize)
    P.check_grads(oracle, h, whole_mu.cpu().numpy(), whole_sg.cpu().numpy(), n, s_total, dsize)


def test_backward_rows_rejects_bad_ranges(hot):
    plan = hot.hot_create(64, 64, 4, 4, 1.0, 0)
    t = torch.zeros(4, 64, device=DEV)
    v = torch.zeros(64, device=DEV)
    rng = hot.hot_rng(seed=1, step=0, first_sample=0)
    with pytest.raises(hot.HotError):
        hot.hot_backward_rows(plan, None, v, v + 1, t[:2], t[:2], 3, False, True, v.clone(), v.clone())     # rows 3..4 of 4
    with pytest.raises(ValueError):
        hot.hot_backward_rows(plan, rng, v, v + 1, t[:2], t[:2], 0, False, True, v.clone(), v.clone())       # both sources
    with pytest.raises(ValueError):
        hot.hot_backward_rows(plan, None, v, v + 1, None, t[:2], 0, False, True, v.clone(), v.clone())       # no source
    hot.hot_destroy(plan)


def test_autograd_wrapper_trains_a_bayesian_mlp(hot):
    """The torch.autograd wrapper: gradients equal fp64 autograd of loss + KL/|D|, and a few Adam steps
    (hot_adam_step) on them lower the loss."""
    from paper_2604_04736_amd.autograd import GaussianSampleLayer
    torch.manual_seed(2)
    d_in, d_h, d_out, batch, s, dsize = 8, 16, 2, 128, 4, 1000.0
    n = d_in * d_h + d_h + d_h * d_out + d_out
    xb = torch.randn(batch, d_in, device=DEV)
    yb = torch.sin(xb[:, :d_out] * 2.0)

    def net_loss(w, x, y):
        o = 0
        w1 = w[o:o + d_in * d_h].view(d_h, d_in); o += d_in * d_h
        b1 = w[o:o + d_h]; o += d_h
        w2 = w[o:o + d_h * d_out].view(d_out, d_h); o += d_h * d_out
        b2 = w[o:o + d_out]
        return ((torch.tanh(x @ w1.T + b1) @ w2.T + b2 - y) ** 2).mean()

    mu = (torch.randn(n, device=DEV) * 0.3).requires_grad_(True)
    sigma = torch.full((n,), 0.05, device=DEV).requires_grad_(True)
    layer = GaussianSampleLayer(n, s, dsize, seed=5)
    w, kl = layer.sample(mu, sigma, step=0)
    loss = sum(net_loss(w[i], xb, yb) for i in range(s)) / s
    loss.backward()
    # reference in fp64 on the CPU with the very same eps
    eps = torch.empty(s, n, device=DEV)
    hot.hot_sample_eps(layer.plan, hot.hot_rng(seed=5, step=0, first_sample=0), eps)
    m64 = mu.detach().double().cpu().requires_grad_(True)
    s64 = sigma.detach().double().cpu().requires_grad_(True)
    e64 = eps.double().cpu()
    ref = sum(net_loss(m64 + s64 * e64[i], xb.double().cpu(), yb.double().cpu()) for i in range(s)) / s
    kl64 = 0.5 * (s64 ** 2 + m64 ** 2 - 1 - 2 * torch.log(s64)).sum()
    (ref + kl64 / dsize).backward()
    assert abs(loss.item() - ref.item()) <= 1e-5 * abs(ref.item())
    assert abs(kl.item() - kl64.item()) <= 1e-7 * abs(kl64.item())
    scale = m64.grad.abs().max().item()
    assert (mu.grad.double().cpu() - m64.grad).abs().max().item() <= 1e-4 * scale
    assert (sigma.grad.double().cpu() - s64.grad).abs().max().item() <= 1e-4 * s64.grad.abs().max().item()
    # a short training run: Adam through the library
    state = [torch.zeros(n, device=DEV) for _ in range(4)]
    first = last = None
    for t in range(1, 61):
        mu.grad = sigma.grad = None
        w, kl = layer.sample(mu, sigma, step=t)
        loss = sum(net_loss(w[i], xb, yb) for i in range(s)) / s
        loss.backward()
        with torch.no_grad():
            hot.hot_adam_step(hot.hot_adam(2e-2, 0.9, 0.999, 1e-8, 1.0, 1e-4, t), mu.data, sigma.data, mu.grad, sigma.grad, *state)
        first = loss.item() if first is None else first
        last = loss.item()
    assert last < 0.5 * first, (first, last)
    assert sigma.min().item() >= 1e-4 * (1 - 1e-6)


def test_any_torch_module_becomes_bayesian(hot):
    """BayesianModule around an nn.Sequential with LayerNorm: the gradients that reach mu and sigma equal
    fp64 autograd of (mean data loss + KL/|D|) with the very same eps, and Adam steps lower the loss."""
    from paper_2604_04736_amd.autograd import BayesianModule
    torch.manual_seed(4)
    net = torch.nn.Sequential(torch.nn.Linear(6, 24), torch.nn.LayerNorm(24), torch.nn.Tanh(), torch.nn.Linear(24, 3)).to(DEV)
    s, dsize = 4, 500.0
    bnn = BayesianModule(net, s, dsize, seed=21)
    n = bnn.mu.numel()
    assert n == sum(p.numel() for p in net.parameters())
    xb = torch.randn(50, 6, device=DEV)
    yb = torch.cos(xb[:, :3])
    out, kl = bnn(xb, step=0)
    assert out.shape == (s, 50, 3)
    loss = ((out - yb[None]) ** 2).mean(dim=(1, 2)).mean()
    loss.backward()

    eps = torch.empty(s, n, device=DEV)
    hot.hot_sample_eps(bnn.layer.plan, hot.hot_rng(seed=21, step=0, first_sample=0), eps)
    m64 = bnn.mu.detach().double().cpu().requires_grad_(True)
    s64 = bnn.sigma.detach().double().cpu().requires_grad_(True)
    net64 = torch.nn.Sequential(torch.nn.Linear(6, 24), torch.nn.LayerNorm(24), torch.nn.Tanh(), torch.nn.Linear(24, 3)).double()
    ref = 0.0
    for i in range(s):
        w = m64 + s64 * eps[i].double().cpu()
        sampled = {name: w[a:b].view(shape) for name, a, b, shape in bnn._slices}
        o = torch.func.functional_call(net64, sampled, (xb.double().cpu(),))
        ref = ref + ((o - yb.double().cpu()) ** 2).mean() / s
    kl64 = 0.5 * (s64 ** 2 + m64 ** 2 - 1 - 2 * torch.log(s64)).sum()
    (ref + kl64 / dsize).backward()
    assert abs(loss.item() - ref.item()) <= 1e-5 * abs(ref.item())
    assert abs(kl.item() - kl64.item()) <= 1e-7 * abs(kl64.item())
    assert (bnn.mu.grad.double().cpu() - m64.grad).abs().max().item() <= 1e-4 * m64.grad.abs().max().item()
    assert (bnn.sigma.grad.double().cpu() - s64.grad).abs().max().item() <= 1e-4 * s64.grad.abs().max().item()

    state = [torch.zeros(n, device=DEV) for _ in range(4)]
    first = last = None
    for t in range(1, 41):
        bnn.mu.grad = bnn.sigma.grad = None
        out, kl = bnn(xb, step=t)
        loss = ((out - yb[None]) ** 2).mean(dim=(1, 2)).mean()
        loss.backward()
        hot.hot_adam_step(hot.hot_adam(1e-2, 0.9, 0.999, 1e-8, 1.0, 1e-5, t), bnn.mu.data, bnn.sigma.data, bnn.mu.grad,
                          bnn.sigma.grad, *state)
        first = loss.item() if first is None else first
        last = loss.item()
    assert last < 0.6 * first, (first, last)
