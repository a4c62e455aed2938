"""Shared pieces of the GPU parity tests: run the HIP path, run the oracle on the very
same bytes, compare element by element with the tolerances stated here.

Tolerances (fp32 path against the fp64 oracle, relative 1e-5 made well-conditioned):
  w          |w - w64|      <= 1e-5 |w64|, and at most 1 ulp from w64 rounded to fp32
             (the kernel uses one fused multiply-add, so it returns the correctly
             rounded exact value);
  KL         |KL - KL64|    <= 1e-5 * 1/2 sum_i (sigma_i^2 + mu_i^2 + 1 + |2 ln sigma_i|);
  grad_mu    |.|            <= 1e-5 (g sum_s |G| + k |mu|);
  grad_sigma |.|            <= 1e-5 (g sum_s |G eps| + k (sigma + 1/sigma)).
The right-hand sides are sums of addend magnitudes: a plain relative error is
meaningless where the addends cancel.
"""
import numpy as np
import torch

RTOL = 1e-5


REDUCE_SUM, REDUCE_MEAN, REDUCE_NONE = 0, 1, 2


def gk(s_local, s_total, dataset_size, reduce_mean=False, flags=None):
    """(g, k) of the gradient and averaging lines for a reduce convention (flags as in hot_desc)."""
    if flags is None:
        flags = REDUCE_MEAN if reduce_mean else REDUCE_SUM
    if flags == REDUCE_NONE:
        return 1.0, 1.0 / dataset_size
    if flags == REDUCE_MEAN:
        return 1.0 / s_local, 1.0 / dataset_size
    return 1.0 / s_total, s_local / (s_total * dataset_size)


def run_hip(hot, x, n, ld, s_local, s_total, dataset_size, flags=0, launch=None, want_kl=True,
            sentinel=None):
    """One forward + backward through the C ABI.  x holds device tensors mu, sigma, eps, G.
    Returns device tensors w (pitch ld, padding prefilled with the sentinel), kl, gmu, gsig."""
    dev = x["mu"].device
    off = (x["mu"].data_ptr() % 16) // 4

    def like(src, fill):
        buf = torch.full((src.numel() + off,), fill, dtype=torch.float32, device=dev)
        return buf[off:].view(src.shape)

    fill = float("nan") if sentinel is None else sentinel
    if x["eps"].shape[1] == ld:
        w = like(x["eps"], fill)
    else:                       # packed [S, N] view of a pitched buffer is not used by the tests
        raise ValueError("eps must be given with its full pitch")
    gmu = like(x["mu"], fill)
    gsig = like(x["mu"], fill)
    kl = torch.full((1,), -1.0, dtype=torch.float64, device=dev) if want_kl else None
    plan = hot.hot_create(n, ld, s_local, s_total, dataset_size, dev.index or 0, flags)
    try:
        if launch:
            for kernel in (hot.HOT_KERNEL_FORWARD, hot.HOT_KERNEL_BACKWARD):
                hot.hot_set_launch(plan, kernel, **launch)
        hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
        hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], gmu, gsig)
        torch.cuda.synchronize()
    finally:
        hot.hot_destroy(plan)
    return w, kl, gmu, gsig


def host(x):
    return {k: np.ascontiguousarray(v.cpu().numpy()) for k, v in x.items()}


def ulp_distance(a32, b32):
    """Distance in units of the last place between two fp32 arrays (finite values)."""
    def key(v):
        i = v.view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7FFFFFFF), i)
    return np.abs(key(np.ascontiguousarray(a32)) - key(np.ascontiguousarray(b32)))


def check_w(oracle, h, w_gpu, n):
    """w_gpu: numpy [S, >=n] fp32."""
    w64 = oracle.reparam(h["mu"], h["sigma"], h["eps"], nthreads=8)
    got = w_gpu[:, :n]
    assert np.all(np.isfinite(got))
    err = np.abs(got.astype(np.float64) - w64)
    assert np.all(err <= RTOL * np.abs(w64)), f"w: max rel err {np.max(err / np.maximum(np.abs(w64), 1e-300))}"
    with np.errstate(over="ignore"):
        ulps = ulp_distance(got, w64.astype(np.float32))
    assert ulps.max() <= 1, f"w: {ulps.max()} ulp from the rounded oracle value"
    return int((ulps > 0).sum())


def kl_scale(h):
    m64, s64 = h["mu"].astype(np.float64), h["sigma"].astype(np.float64)
    return 0.5 * float(np.sum(s64 * s64 + m64 * m64 + 1.0 + np.abs(2.0 * np.log(s64))))


def check_kl(oracle, h, kl_gpu):
    want = oracle.kl(h["mu"], h["sigma"])
    scale = kl_scale(h)
    assert abs(kl_gpu - want) <= RTOL * scale, f"KL {kl_gpu} vs {want}, scale {scale}"
    return abs(kl_gpu - want) / scale


def check_grads(oracle, h, gmu_gpu, gsig_gpu, n, s_total, dataset_size, reduce_mean=False, flags=None):
    """flags = HOT_REDUCE_NONE: the oracle's mean convention is g = 1/S_loc, k = 1/|D|; called on ONE sample
    at a time (g = 1) and summed over the samples with the KL part counted once, it is the definition of
    the unscaled convention g = 1, k = 1/|D| (the gradient is linear in G)."""
    s_local = h["eps"].shape[0]
    if flags is None:
        flags = REDUCE_MEAN if reduce_mean else REDUCE_SUM
    if flags == REDUCE_NONE:
        gm64, gs64 = np.zeros(n), np.zeros(n)
        for s in range(s_local):
            a, b = oracle.grad(h["mu"], h["sigma"], np.ascontiguousarray(h["eps"][s:s + 1]),
                               np.ascontiguousarray(h["G"][s:s + 1]), 1, dataset_size, True, nthreads=8)
            gm64 += a
            gs64 += b
        if s_local > 1:       # each of the S_loc calls added the KL part k * mu, k * (sigma - 1/sigma) once
            z = np.zeros((1, h["eps"].shape[1]), np.float32)
            a, b = oracle.grad(h["mu"], h["sigma"], z, z, 1, dataset_size, True, nthreads=8)
            gm64 -= (s_local - 1) * a
            gs64 -= (s_local - 1) * b
    else:
        gm64, gs64 = oracle.grad(h["mu"], h["sigma"], h["eps"], h["G"], s_total, dataset_size,
                                 flags == REDUCE_MEAN, nthreads=8)
    g, k = gk(s_local, s_total, dataset_size, flags=flags)
    m64, s64 = h["mu"].astype(np.float64), h["sigma"].astype(np.float64)
    sum_abs_g = np.zeros(n)
    sum_abs_ge = np.zeros(n)
    for s in range(s_local):
        G64 = h["G"][s, :n].astype(np.float64)
        sum_abs_g += np.abs(G64)
        sum_abs_ge += np.abs(G64 * h["eps"][s, :n].astype(np.float64))
    tol_mu = RTOL * (g * sum_abs_g + k * np.abs(m64))
    tol_sg = RTOL * (g * sum_abs_ge + k * (s64 + 1.0 / s64))
    err_mu = np.abs(gmu_gpu.astype(np.float64) - gm64)
    err_sg = np.abs(gsig_gpu.astype(np.float64) - gs64)
    assert np.all(err_mu <= tol_mu), f"grad_mu: worst {np.max(err_mu / np.maximum(tol_mu, 1e-300)) * RTOL} of scale"
    assert np.all(err_sg <= tol_sg), f"grad_sigma: worst {np.max(err_sg / np.maximum(tol_sg, 1e-300)) * RTOL} of scale"
    return float(np.max(err_mu / np.maximum(tol_mu, 1e-300)) * RTOL), \
        float(np.max(err_sg / np.maximum(tol_sg, 1e-300)) * RTOL)


def check_all(oracle, hot, x, wl, launch=None, flags=0, sentinel=123456.0):
    """Full element-by-element comparison of one workload; returns a small report."""
    n, ld = wl.n_weights, wl.ld
    w, kl, gmu, gsig = run_hip(hot, x, n, ld, wl.s_local, wl.s_total, wl.dataset_size, flags,
                               launch, True, sentinel)
    h = host(x)
    wh = w.cpu().numpy()
    if ld > n:
        assert np.all(wh[:, n:] == np.float32(sentinel)), "w padding was written"
    rep = {"w_inexact": check_w(oracle, h, wh, n)}
    rep["kl_rel"] = check_kl(oracle, h, kl.item())
    rep["gmu_rel"], rep["gsig_rel"] = check_grads(oracle, h, gmu.cpu().numpy(), gsig.cpu().numpy(), n,
                                                  wl.s_total, wl.dataset_size, flags=flags)
    return rep


def check_all_chunked(oracle, hot, x, wl, chunk=1 << 24, say=None):
    """check_all for workloads whose fp64 oracle outputs should not sit in host memory all at once: the HIP
    path runs once over the whole workload (default launch shape), then every element of w, grad_mu and
    grad_sigma is compared with the oracle column block by column block, and the KL term over all weights."""
    n, ld = wl.n_weights, wl.ld
    w, kl, gmu, gsig = run_hip(hot, x, n, ld, wl.s_local, wl.s_total, wl.dataset_size, 0, None, True, 123456.0)
    if ld > n:
        assert bool((w[:, n:] == 123456.0).all()), "w padding was written"
    rep = {"kl_rel": check_kl(oracle, {"mu": x["mu"].cpu().numpy(), "sigma": x["sigma"].cpu().numpy()}, kl.item()),
           "w_inexact": 0, "gmu_rel": 0.0, "gsig_rel": 0.0, "blocks": 0}
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        h = {"mu": x["mu"][a:b].cpu().numpy(), "sigma": x["sigma"][a:b].cpu().numpy(),
             "eps": np.ascontiguousarray(x["eps"][:, a:b].cpu().numpy()),
             "G": np.ascontiguousarray(x["G"][:, a:b].cpu().numpy())}
        rep["w_inexact"] += check_w(oracle, h, w[:, a:b].cpu().numpy(), b - a)
        gm, gs = check_grads(oracle, h, gmu[a:b].cpu().numpy(), gsig[a:b].cpu().numpy(), b - a,
                             wl.s_total, wl.dataset_size)
        rep["gmu_rel"], rep["gsig_rel"] = max(rep["gmu_rel"], gm), max(rep["gsig_rel"], gs)
        rep["blocks"] += 1
        if say:
            say("block", a, b, "ok")
    return rep
