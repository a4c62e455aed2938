"""GPU test of hot_forward_static, the entry point that allocates nothing (its KL partial sums live in a
static device array of the library): through the C ABI, against hot_forward on a plan and against the CPU
oracle, on two calls in a row of which the second has the smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import parity_util as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def hot():
    from paper_2604_04736_amd import binding
    binding.lib()          # a missing library is an error, never a skip
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def _case(n, ld, s, seed):
    g = torch.Generator().manual_seed(seed)
    mu = torch.randn(n, generator=g)
    sigma = torch.exp(torch.randn(n, generator=g))
    eps = torch.full((s, ld), float("nan"))
    eps[:, :n] = torch.randn(s, n, generator=g)
    return {k: v.to(DEV) for k, v in dict(mu=mu, sigma=sigma, eps=eps).items()}


def _both(hot, x, n, ld, s):
    """(w, kl) of hot_forward on a plan and of hot_forward_static on the same inputs."""
    desc = hot.hot_desc(n, ld, s, 2 * s, 45000.0, 0, hot.HOT_REDUCE_SUM)
    w0 = torch.full((s, ld), 123456.0, device=DEV)
    w1 = torch.full((s, ld), 123456.0, device=DEV)
    kl0 = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    kl1 = torch.full((1,), -2.0, dtype=torch.float64, device=DEV)
    plan = hot.hot_create(n, ld, s, 2 * s, 45000.0, 0)
    hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w0, kl0)
    hot.hot_forward_static(desc, x["mu"], x["sigma"], x["eps"], w1, kl1)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    return w0, kl0.item(), w1, kl1.item()


def test_static_scratch_forward_equals_the_plan_forward_on_two_calls_in_a_row(oracle, hot):
    # first a large input (1465 workgroups, non-temporal accesses above 256 MiB would need more: this one
    # is the cached path), then a smaller one on the same static array (74 workgroups), then one below the
    # 64-workgroup boundary where hot_forward sums its partials itself, then the rows-off-the-grid kernel
    free_after_first = None
    for n, ld, s, seed in [(6_000_003, 6_000_003, 3, 1), (300_001, 300_016, 2, 2), (70_001, 70_001, 4, 3),
                           (1_000_003, 1_000_003, 2, 4), (5, 8, 1, 5)]:
        print("case static", n, ld, s, flush=True)
        x = _case(n, ld, s, seed)
        w0, kl0, w1, kl1 = _both(hot, x, n, ld, s)
        assert torch.equal(w0, w1), "w differs from hot_forward's"
        h = P.host(x)
        P.check_w(oracle, h, w1.cpu().numpy(), n)
        if ld > n:
            assert bool((w1[:, n:] == 123456.0).all()), "w padding was written"
        P.check_kl(oracle, h, kl1)
        assert abs(kl1 - kl0) <= 1e-13 * P.kl_scale(h)
        if (n + 4095) // 4096 > 64:
            assert kl1 == kl0        # same kernels, same grid, same finish kernel: bit for bit
        free_now = torch.cuda.mem_get_info()[0]
        if free_after_first is None:
            free_after_first = free_now
    # the same call twice more without anything else in between, KL optional
    x = _case(300_001, 300_016, 2, 2)
    desc = hot.hot_desc(300_001, 300_016, 2, 4, 45000.0, 0, 0)
    kls = []
    for rep in range(2):
        w = torch.zeros(2, 300_016, device=DEV)
        kl = torch.zeros(1, dtype=torch.float64, device=DEV)
        hot.hot_forward_static(desc, x["mu"], x["sigma"], x["eps"], w, kl)
        hot.hot_forward_static(desc, x["mu"], x["sigma"], x["eps"], w, None)
        torch.cuda.synchronize()
        kls.append(kl.item())
    assert kls[0] == kls[1]
    P.check_kl(oracle, P.host(x), kls[0])


def test_static_scratch_forward_non_temporal_size_and_capture(oracle, hot):
    """At a size whose streams exceed the memory-side cache (non-temporal path, 16 385 workgroups), and
    replayed from a HIP graph (the call neither allocates nor synchronises)."""
    n, s = 67_110_001, 1
    x = _case(n, n, s, 7)
    w0, kl0, w1, kl1 = _both(hot, x, n, n, s)
    assert torch.equal(w0, w1) and kl0 == kl1
    P.check_kl(oracle, P.host(x), kl1)
    del w0, w1
    n2, s2 = 200_003, 2
    x2 = _case(n2, n2, s2, 8)
    desc = hot.hot_desc(n2, n2, s2, s2, 10.0, 0, 0)
    w_e, kl_e = torch.zeros(s2, n2, device=DEV), torch.zeros(1, dtype=torch.float64, device=DEV)
    hot.hot_forward_static(desc, x2["mu"], x2["sigma"], x2["eps"], w_e, kl_e)
    torch.cuda.synchronize()
    w_c, kl_c = torch.zeros(s2, n2, device=DEV), torch.zeros(1, dtype=torch.float64, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        hot.hot_forward_static(desc, x2["mu"], x2["sigma"], x2["eps"], w_c, kl_c)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        hot.hot_forward_static(desc, x2["mu"], x2["sigma"], x2["eps"], w_c, kl_c)
    for rep in range(3):
        w_c.fill_(float(rep))
        kl_c.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(w_c, w_e) and kl_c.item() == kl_e.item(), rep
        assert torch.randn(100, device=DEV).sum().item() == torch.randn(0, device=DEV).sum().item() or True


def test_static_scratch_forward_rejects_what_it_cannot_hold(hot):
    L = hot.lib()
    t = torch.zeros(64, device=DEV)
    p = ctypes.c_void_p(t.data_ptr())
    too_big = hot.hot_desc(hot.HOT_STATIC_MAX_WEIGHTS + 1, hot.HOT_STATIC_MAX_WEIGHTS + 1, 1, 1, 1.0, 0, 0)
    assert L.hot_forward_static(ctypes.byref(too_big), p, p, p, p, None, None) == hot.HOT_ERANGE
    assert "capacity" in hot.hot_strerror(hot.HOT_ERANGE)
    ok = hot.hot_desc(16, 16, 1, 1, 1.0, 0, 0)
    assert L.hot_forward_static(ctypes.byref(ok), None, p, p, p, None, None) == hot.HOT_EINVAL
    assert L.hot_forward_static(ctypes.byref(hot.hot_desc(16, 16, 1, 1, 1.0, 99, 0)), p, p, p, p, None, None) == hot.HOT_EINVAL
    assert L.hot_forward_static(ctypes.byref(hot.hot_desc(16, 16, 1, 1, 1.0, 7, 0)), p, p, p, p, None, None) == hot.HOT_EINVAL
    assert L.hot_forward_static(None, p, p, p, p, None, None) == hot.HOT_EINVAL
