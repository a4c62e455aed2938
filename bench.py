#!/usr/bin/env python3
"""Benchmark of the libhot hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: hot_forward
(reparameterisation + KL term) followed by hot_backward (sample-gradient reduction),
i.e. what one GPU does per training step of Algorithm 2 around the network's own
forward/backward.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-job items/s (an item is one (sample, weight) pair), the
roofline of the dominant kernel from HIP-event timings taken inside the timed region,
and the CPU oracle timed on the host as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
METRIC = "hot-path items/sec on 1 MI355X + % of HBM-BW or MFMA roofline"


def algorithmic_bytes(n: int, s: int, in_kernel_eps: bool = False):
    """Bytes the method must move per launch (fp32): eps read from its array, or drawn in registers."""
    e = 0 if in_kernel_eps else 4 * s * n
    fwd = e + 4 * 2 * n + 4 * s * n + 8                # [eps,] mu, sigma in; w, KL out
    bwd = 4 * s * n + e + 4 * 2 * n + 4 * 2 * n        # G, [eps,] mu, sigma in; grad_mu, grad_sigma out
    return fwd, bwd


RNG_SEED, RNG_STEP = 0x5EED, 1


def time_steps(hot, torch, wl, x, steps: int, warmup: int, in_kernel_eps: bool = False):
    dev = x["mu"].device
    w = torch.empty_like(x["G"])
    kl = torch.zeros(1, dtype=torch.float64, device=dev)
    gmu = torch.empty_like(x["mu"])
    gsig = torch.empty_like(x["mu"])
    plan = hot.hot_create(wl.n_weights, wl.ld, wl.s_local, wl.s_total, wl.dataset_size, dev.index or 0)
    rng = hot.hot_rng(seed=RNG_SEED, step=RNG_STEP, first_sample=0)

    def step(events=None):
        if events is not None:
            events[0].record()
        if in_kernel_eps:
            hot.hot_forward_rng(plan, rng, x["mu"], x["sigma"], w, kl)
        else:
            hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
        if events is not None:
            events[1].record()
        if in_kernel_eps:
            hot.hot_backward_rng(plan, rng, x["mu"], x["sigma"], x["G"], gmu, gsig)
        else:
            hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], gmu, gsig)
        if events is not None:
            events[2].record()

    for _ in range(warmup):
        step()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fwd_all = sorted(e[0].elapsed_time(e[1]) for e in ev)
    bwd_all = sorted(e[1].elapsed_time(e[2]) for e in ev)
    fwd_ms, bwd_ms = sum(fwd_all) / steps, sum(bwd_all) / steps
    spread = {"fwd_median_ms": fwd_all[steps // 2], "fwd_min_ms": fwd_all[0],
              "bwd_median_ms": bwd_all[steps // 2], "bwd_min_ms": bwd_all[0]}
    launch = {"forward": hot.hot_get_launch(plan, hot.HOT_KERNEL_FORWARD_RNG if in_kernel_eps else hot.HOT_KERNEL_FORWARD),
              "backward": hot.hot_get_launch(plan, hot.HOT_KERNEL_BACKWARD_RNG if in_kernel_eps else hot.HOT_KERNEL_BACKWARD)}
    hot.hot_destroy(plan)
    return {"wall_s": wall, "fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "spread": spread, "launch": launch,
            "out": {"w": w, "kl": kl, "gmu": gmu, "gsig": gsig}}


def time_kernels_between_other_work(hot, torch, wl, x, iters: int = 20, in_kernel_eps: bool = False, plain: bool = False):
    """ms of each kernel when an unrelated element-wise kernel (512 MiB read and written with plain accesses: a
    stand-in for the network that runs between the two calls in training) precedes it, so that the memory-side
    cache holds somebody else's partly dirty lines instead of this library's arrays.  plain: the same with the
    library's non-temporal hints switched off."""
    dev = x["mu"].device
    other = torch.zeros(128 << 20, dtype=torch.float32, device=dev)
    w = torch.empty_like(x["G"])
    kl = torch.zeros(1, dtype=torch.float64, device=dev)
    gmu, gsig = torch.empty_like(x["mu"]), torch.empty_like(x["mu"])
    plan = hot.hot_create(wl.n_weights, wl.ld, wl.s_local, wl.s_total, wl.dataset_size, dev.index or 0)
    if plain:
        for kern in (hot.HOT_KERNEL_FORWARD, hot.HOT_KERNEL_BACKWARD, hot.HOT_KERNEL_FORWARD_RNG, hot.HOT_KERNEL_BACKWARD_RNG):
            hot.hot_set_launch(plan, kern, nontemporal=0)
    rng = hot.hot_rng(seed=RNG_SEED, step=RNG_STEP, first_sample=0)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(iters)]
    for i in range(3 + iters):
        e = ev[i - 3] if i >= 3 else None
        other.add_(1.0)
        if e:
            e[0].record()
        if in_kernel_eps:
            hot.hot_forward_rng(plan, rng, x["mu"], x["sigma"], w, kl)
        else:
            hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
        if e:
            e[1].record()
        other.add_(1.0)
        if e:
            e[2].record()
        if in_kernel_eps:
            hot.hot_backward_rng(plan, rng, x["mu"], x["sigma"], x["G"], gmu, gsig)
        else:
            hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], gmu, gsig)
        if e:
            e[3].record()
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    f = sorted(e[0].elapsed_time(e[1]) for e in ev)
    b = sorted(e[2].elapsed_time(e[3]) for e in ev)
    del other, w
    torch.cuda.empty_cache()
    return {"fwd_ms": f[iters // 2], "bwd_ms": b[iters // 2]}


def between_other_work(hot, torch, wl, x, in_kernel_eps: bool):
    hinted = time_kernels_between_other_work(hot, torch, wl, x, 20, in_kernel_eps, False)
    plain = time_kernels_between_other_work(hot, torch, wl, x, 20, in_kernel_eps, True)
    fb, bb = algorithmic_bytes(wl.n_weights, wl.s_local, in_kernel_eps)
    return {"fwd_ms": hinted["fwd_ms"], "bwd_ms": hinted["bwd_ms"],
            "fwd_GBps": fb / hinted["fwd_ms"] / 1e6, "bwd_GBps": bb / hinted["bwd_ms"] / 1e6,
            "kernels_frac_of_hbm_roofline": (fb + bb) / ((hinted["fwd_ms"] + hinted["bwd_ms"]) * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "with_plain_accesses": plain,
            "what": "each kernel timed right after an unrelated 512 MiB element-wise kernel (the network's stand-in); "
                    "with_plain_accesses: the same with the non-temporal hints switched off"}


def time_graph_steps(hot, torch, wl, x, steps: int, in_kernel_eps: bool = False) -> float:
    """ms per step when the step (forward, KL finish, backward) is captured once in a HIP graph and
    replayed: what a launch-latency-bound small workload costs without the host in the loop."""
    dev = x["mu"].device
    w = torch.empty_like(x["G"])
    kl = torch.zeros(1, dtype=torch.float64, device=dev)
    gmu, gsig = torch.empty_like(x["mu"]), torch.empty_like(x["mu"])
    plan = hot.hot_create(wl.n_weights, wl.ld, wl.s_local, wl.s_total, wl.dataset_size, dev.index or 0)
    rng = hot.hot_rng(seed=RNG_SEED, step=RNG_STEP, first_sample=0)

    def step():
        if in_kernel_eps:
            hot.hot_forward_rng(plan, rng, x["mu"], x["sigma"], w, kl)
            hot.hot_backward_rng(plan, rng, x["mu"], x["sigma"], x["G"], gmu, gsig)
        else:
            hot.hot_forward(plan, x["mu"], x["sigma"], x["eps"], w, kl)
            hot.hot_backward(plan, x["mu"], x["sigma"], x["eps"], x["G"], gmu, gsig)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    del graph
    hot.hot_destroy(plan)
    return ms


def verify_sampled(oracle, np, wl, x, out, blocks: int = 6, width: int = 20_000, in_kernel_eps: bool = False) -> bool:
    """Checks the timed buffers on a few column blocks against the oracle (same tolerances as the tests)."""
    if in_kernel_eps:
        return verify_sampled_rng(oracle, np, wl, x, out, blocks, width)
    n = wl.n_weights
    rng = np.random.default_rng(wl.seed)
    spans = [(0, min(width, n)), (max(0, n - width), n)]
    spans += [(a, min(n, a + width)) for a in rng.integers(0, max(1, n - width), size=blocks)]
    g = 1.0 / wl.s_total
    k = wl.s_local / (wl.s_total * wl.dataset_size)
    for a, b in spans:
        a, b = int(a), int(b)
        mu = x["mu"][a:b].cpu().numpy()
        sg = x["sigma"][a:b].cpu().numpy()
        eps = np.ascontiguousarray(x["eps"][:, a:b].cpu().numpy())
        G = np.ascontiguousarray(x["G"][:, a:b].cpu().numpy())
        w64 = oracle.reparam(mu, sg, eps)
        if not np.all(np.abs(out["w"][:, a:b].cpu().numpy() - w64) <= 1e-5 * np.abs(w64)):
            return False
        gm64, gs64 = oracle.grad(mu, sg, eps, G, wl.s_total, wl.dataset_size)
        G64, e64, m64, s64 = G.astype(np.float64), eps.astype(np.float64), mu.astype(np.float64), sg.astype(np.float64)
        if not np.all(np.abs(out["gmu"][a:b].cpu().numpy() - gm64) <= 1e-5 * (g * np.abs(G64).sum(0) + k * np.abs(m64))):
            return False
        if not np.all(np.abs(out["gsig"][a:b].cpu().numpy() - gs64)
                      <= 1e-5 * (g * np.abs(G64 * e64).sum(0) + k * (s64 + 1 / s64))):
            return False
    return True


def verify_sampled_rng(oracle, np, wl, x, out, blocks: int, width: int) -> bool:
    """Same for the in-kernel draw: the oracle draws its own eps (fp64) for the sampled windows."""
    n = wl.n_weights
    rng = np.random.default_rng(wl.seed)
    spans = [(0, min(width, n)), (max(0, n - width), n)]
    spans += [(a, min(n, a + width)) for a in rng.integers(0, max(1, n - width), size=blocks)]
    g = 1.0 / wl.s_total
    k = wl.s_local / (wl.s_total * wl.dataset_size)
    for a, b in spans:
        a, b = int(a), int(b)
        m64 = x["mu"][a:b].cpu().numpy().astype(np.float64)
        s64 = x["sigma"][a:b].cpu().numpy().astype(np.float64)
        G64 = x["G"][:, a:b].cpu().numpy().astype(np.float64)
        e64, r64 = oracle.eps_normal(b - a, wl.s_local, RNG_SEED, RNG_STEP, 0, with_radius=True, col0=a)
        w64 = m64 + s64 * e64
        if not np.all(np.abs(out["w"][:, a:b].cpu().numpy() - w64) <= 1e-5 * (np.abs(m64) + s64 * r64)):
            return False
        gm64 = g * G64.sum(0) + k * m64
        gs64 = g * (G64 * e64).sum(0) + k * (s64 - 1 / s64)
        if not np.all(np.abs(out["gmu"][a:b].cpu().numpy() - gm64) <= 1e-5 * (g * np.abs(G64).sum(0) + k * np.abs(m64))):
            return False
        if not np.all(np.abs(out["gsig"][a:b].cpu().numpy() - gs64)
                      <= 1e-5 * (g * (np.abs(G64) * (np.abs(e64) + r64)).sum(0) + k * (s64 + 1 / s64))):
            return False
    return True


def compare_every_element(np, wl, h, n, w64, kl64, gm64, gs64, out):
    """Every element of the timed buffers against the oracle arrays cpu_baseline has just computed: the
    largest error of each output in units of its tolerance scale (the tests' scales: |w64| for w, the sums
    of addend magnitudes for the KL term and the gradients) and whether all lie within 1e-5 of it."""
    g = 1.0 / wl.s_total
    k = wl.s_local / (wl.s_total * wl.dataset_size)
    worst = {"w": 0.0, "grad_mu": 0.0, "grad_sigma": 0.0}
    step = 1 << 24
    tiny = np.finfo(np.float64).tiny
    for a in range(0, n, step):
        b = min(n, a + step)
        m64, s64 = h["mu"][a:b].astype(np.float64), h["sigma"][a:b].astype(np.float64)
        G64, e64 = h["G"][:, a:b].astype(np.float64), h["eps"][:, a:b].astype(np.float64)
        ref = w64[:, a:b]
        err = np.abs(out["w"][:, a:b].cpu().numpy() - ref) / np.maximum(np.abs(ref), tiny)
        worst["w"] = max(worst["w"], float(err.max()))
        scale = g * np.abs(G64).sum(0) + k * np.abs(m64)
        err = np.abs(out["gmu"][a:b].cpu().numpy() - gm64[a:b]) / np.maximum(scale, tiny)
        worst["grad_mu"] = max(worst["grad_mu"], float(err.max()))
        scale = g * np.abs(G64 * e64).sum(0) + k * (s64 + 1.0 / s64)
        err = np.abs(out["gsig"][a:b].cpu().numpy() - gs64[a:b]) / np.maximum(scale, tiny)
        worst["grad_sigma"] = max(worst["grad_sigma"], float(err.max()))
    m64, s64 = h["mu"].astype(np.float64), h["sigma"].astype(np.float64)
    kl_scale = 0.5 * float(np.sum(s64 * s64 + m64 * m64 + 1.0 + np.abs(2.0 * np.log(s64))))
    worst["kl"] = abs(out["kl"].item() - kl64) / kl_scale
    return {"max_error_over_scale": worst, "tolerance": 1e-5, "elements": {"w": n * wl.s_local, "grad_mu": n, "grad_sigma": n},
            "all_within_tolerance": bool(all(v <= 1e-5 for v in worst.values())),
            "scales": "w: |w64|; KL: 1/2 sum(sigma^2 + mu^2 + 1 + |2 ln sigma|); grad_mu: g sum_s|G| + k|mu|; "
                      "grad_sigma: g sum_s|G eps| + k(sigma + 1/sigma)"}


def cpu_baseline(oracle, np, wl, x, max_weights: int, out=None):
    """The oracle as it stands, timed on the host cores over the first max_weights weights.  With the timed
    buffers in `out` and the whole workload inside max_weights, the arrays the oracle has just produced are
    then compared with them element by element (outside the timed interval)."""
    n = min(wl.n_weights, max_weights)
    # the threads the oracle is given: the cores this process may run on, within OMP_NUM_THREADS when the
    # environment sets a CPU share (the GPU machines do: 16 per GPU, whatever the host's core count)
    host_cores = os.cpu_count() or 1
    affinity = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else host_cores
    share = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    cores = max(1, min(affinity, share) if share > 0 else affinity)
    h = {"mu": x["mu"][:n].cpu().numpy(), "sigma": x["sigma"][:n].cpu().numpy(),
         "eps": np.ascontiguousarray(x["eps"][:, :n].cpu().numpy()),
         "G": np.ascontiguousarray(x["G"][:, :n].cpu().numpy())}
    used = oracle.threads(cores)
    t0 = time.perf_counter()
    w64 = oracle.reparam(h["mu"], h["sigma"], h["eps"], used)
    kl64 = oracle.kl(h["mu"], h["sigma"])
    gm, gs = oracle.grad(h["mu"], h["sigma"], h["eps"], h["G"], wl.s_total, wl.dataset_size, False, used)
    dt = time.perf_counter() - t0
    compared = None
    if out is not None and n == wl.n_weights:
        compared = compare_every_element(np, wl, h, n, w64, kl64, gm, gs, out)
    del w64, gm, gs
    # the same three calls on one thread, over an eighth of the sample
    n1 = max(1, n // 8)
    h1 = {"mu": h["mu"][:n1], "sigma": h["sigma"][:n1], "eps": np.ascontiguousarray(h["eps"][:, :n1]),
          "G": np.ascontiguousarray(h["G"][:, :n1])}
    one = oracle.threads(1)
    t1 = time.perf_counter()
    w64 = oracle.reparam(h1["mu"], h1["sigma"], h1["eps"], one)
    oracle.kl(h1["mu"], h1["sigma"])
    gm, gs = oracle.grad(h1["mu"], h1["sigma"], h1["eps"], h1["G"], wl.s_total, wl.dataset_size, False, one)
    dt1 = time.perf_counter() - t1
    del w64, gm, gs
    return {"value": n * wl.s_local / dt, "unit": "items/s", "cores": used, "kind": "oracle",
            "host": {"nproc": host_cores, "affinity": affinity, "omp_num_threads_env": share or None},
            "single_thread": {"value": n1 * wl.s_local / dt1, "unit": "items/s", "cores": one,
                              "sample": f"first {n1} weights, {dt1:.1f} s"},
            "sample": f"first {n} of {wl.n_weights} weights x {wl.s_local} samples of {wl.name}, "
                      f"forward + KL + backward, {dt:.1f} s (KL sum is serial by definition)",
            "kl": kl64, "every_element": compared}


def alu_roofline_forward_rng(workload: str, achieved_items_per_s: float):
    """Vector-ALU ceiling of the drawing forward kernel from hardware counters (the committed rocprofv3 summary
    of this workload): SQ_ACTIVE_INST_VALU gives the SIMD-cycles the vector ALUs were busy per launch, hence per
    item; the chip has 1024 SIMDs (256 compute units x 4) at a nominal 2.4 GHz, so at most
    1024 * 2.4e9 / (SIMD-cycles per item) items/s.  The summary also holds the clock the chip actually ran the
    kernel at (GRBM_GUI_ACTIVE per XCD over the kernel's duration) and the busy fraction at that clock."""
    path = os.path.join(ROOT, "profiles", f"hot_forward_rng_kernel_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None
    text = open(path).read()

    def field(name):
        m = re.search(r"^" + name + r":\s*([0-9.eE+-]+)", text, re.M)
        return float(m.group(1)) if m else None

    per_item, clock, busy = field("valu_simd_cycles_per_item"), field("measured_clock_GHz"), field("valu_busy_frac_at_measured_clock")
    if per_item is None:
        return None
    peak = 1024 * 2.4e9 / per_item
    return {"bound": "alu", "kernel": "hot_forward_kernel (drawn eps)", "achieved": achieved_items_per_s, "peak": peak,
            "unit": "items/s", "frac": achieved_items_per_s / peak, "valu_simd_cycles_per_item": per_item,
            "measured_clock_GHz": clock, "valu_busy_frac_at_measured_clock": busy,
            "source": "SQ_ACTIVE_INST_VALU, GRBM_GUI_ACTIVE of " + os.path.basename(path)}


def framework_step(torch, wl, x, iters: int = 5):
    """The same step written with stock PyTorch operators on the same GPU (the software the paper's own
    experiments ran on): w = addcmul(mu, sigma, eps), the KL expression in fp32, and the column reductions of
    G and G * eps with the KL gradient.  Context for the figures above, not a target."""
    mu, sigma, eps, G = x["mu"], x["sigma"], x["eps"][:, :wl.n_weights], x["G"][:, :wl.n_weights]
    g = 1.0 / wl.s_total
    k = wl.s_local / (wl.s_total * wl.dataset_size)

    def step():
        w = torch.addcmul(mu, sigma, eps)
        kl = 0.5 * (sigma * sigma + mu * mu - 1.0 - 2.0 * torch.log(sigma)).sum(dtype=torch.float64)
        gmu = torch.add(G.sum(0), mu, alpha=k / g).mul_(g)
        gsig = torch.add((G * eps).sum(0), sigma - 1.0 / sigma, alpha=k / g).mul_(g)
        return w, kl, gmu, gsig

    for _ in range(2):
        step()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        out = step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    del out
    torch.cuda.empty_cache()
    return {"ms_per_step": ms, "items_per_s": wl.items / (ms * 1e-3),
            "what": "torch.addcmul + KL expression in fp32 (fp64 sum) + G.sum(0), (G * eps).sum(0) with the KL gradient, eager mode"}


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def copy_ceiling(hot, torch, dev, nbytes: int = 1 << 31, iters: int = 20, nontemporal: int = 1):
    """GB/s (bytes read + bytes written) of the library's plain copy kernel over nbytes."""
    src = torch.empty(nbytes // 4, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        hot.hot_probe_copy(dst, src, nontemporal)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        hot.hot_probe_copy(dst, src, nontemporal)
    e1.record()
    torch.cuda.synchronize()
    ok = bool(torch.equal(dst, src))
    ms = e0.elapsed_time(e1) / iters
    # an independent witness of what this machine's memory system gives a copy: the HIP runtime's own
    # device-to-device copy (torch's copy_ of a contiguous tensor) over the same buffers
    for _ in range(3):
        dst.copy_(src)
    e0.record()
    for _ in range(iters):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms_rt = e0.elapsed_time(e1) / iters
    return {"GBps": 2 * nbytes / ms / 1e6, "ms": ms, "bytes_read": nbytes, "bytes_written": nbytes,
            "nontemporal": nontemporal, "copied_correctly": ok, "runtime_copy_GBps": 2 * nbytes / ms_rt / 1e6}


def mix_ceiling(hot, torch, dev, stream_bytes: int, reads: int, writes: int, iters: int = 20):
    """GB/s of a no-arithmetic kernel with the given numbers of equally long read and write streams."""
    arena = torch.empty((reads + writes) * stream_bytes // 4, dtype=torch.float32, device=dev)
    arena[: reads * stream_bytes // 4].normal_()
    for _ in range(3):
        hot.hot_probe_streams(arena, stream_bytes, reads, writes)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        hot.hot_probe_streams(arena, stream_bytes, reads, writes)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    return {"GBps": (reads + writes) * stream_bytes / ms / 1e6, "ms": ms, "read_streams": reads,
            "write_streams": writes, "stream_bytes": stream_bytes}


def stream_mix(wl, in_kernel_eps: bool):
    """(read streams, write streams) of N floats each that the two kernels move: forward reads (the eps rows,) mu,
    sigma and writes the w rows; backward reads the G rows (and the eps rows), mu, sigma and writes grad_mu, grad_sigma."""
    rows = wl.s_local
    return {"forward": ((0 if in_kernel_eps else rows) + 2, rows), "backward": ((1 if in_kernel_eps else 2) * rows + 2, 2)}


def mix_ceilings(hot, torch, dev, wl, in_kernel_eps: bool, fwd_ms: float, bwd_ms: float):
    """Both kernels of a workload beside hot_probe_streams with their stream counts (no arithmetic)."""
    out = {}
    fb, bb = algorithmic_bytes(wl.n_weights, wl.s_local, in_kernel_eps)
    # the probe's streams lie as the workload's rows do: at its pitch, off the 16-byte grid where that is (C5)
    stream_bytes = 4 * wl.ld
    for which, (r, w), nbytes, ms in (("forward",) + (stream_mix(wl, in_kernel_eps)["forward"],) + (fb, fwd_ms),
                                      ("backward",) + (stream_mix(wl, in_kernel_eps)["backward"],) + (bb, bwd_ms)):
        if r > 64 or w > 64:
            continue
        m = mix_ceiling(hot, torch, dev, stream_bytes, r, w)
        out[which] = {"probe_GBps": m["GBps"], "probe_ms": m["ms"], "read_streams": r, "write_streams": w,
                      "stream_bytes": stream_bytes, "kernel_GBps": nbytes / ms / 1e6, "kernel_vs_probe": nbytes / ms / 1e6 / m["GBps"]}
        if stream_bytes % 16:
            a = mix_ceiling(hot, torch, dev, stream_bytes // 16 * 16, r, w)
            out[which]["probe_on_the_16_byte_grid_GBps"] = a["GBps"]
            out[which]["kernel_vs_probe_on_the_16_byte_grid"] = nbytes / ms / 1e6 / a["GBps"]
        torch.cuda.empty_cache()
    return out


def predictive_stats_lines(hot, torch, dev, iters: int = 20):
    """hot_stats_local + hot_stats_merge on the prediction shapes of the paper's three use cases
    (samples x (batch x outputs)) and on one large synthetic shape that leaves the caches."""
    out = {}
    shapes = {"vit_16x(256x10)": (16, 256 * 10), "mlp_16x(64x24)": (16, 64 * 24),
              "swin_2x(69x121x240)": (2, 69 * 121 * 240), "synthetic_16x2^24": (16, 1 << 24)}
    for name, (s, m) in shapes.items():
        y = torch.randn(s, m, device=dev)
        mean = torch.empty(m, dtype=torch.float64, device=dev)
        m2 = torch.empty_like(mean)
        mo, so = torch.empty(m, device=dev), torch.empty(m, device=dev)

        def run():
            hot.hot_stats_local(y, mean, m2)
            hot.hot_stats_merge(mean.view(1, m), m2.view(1, m), [s], 1, mo, so)

        for _ in range(3):
            run()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ms_l = ms_m = 0.0
        for _ in range(iters):
            e[0].record()
            hot.hot_stats_local(y, mean, m2)
            e[1].record()
            hot.hot_stats_merge(mean.view(1, m), m2.view(1, m), [s], 1, mo, so)
            e[2].record()
            torch.cuda.synchronize()
            ms_l += e[0].elapsed_time(e[1]) / iters
            ms_m += e[1].elapsed_time(e[2]) / iters
        ok = bool(torch.allclose(mo, y.mean(0), rtol=1e-5, atol=1e-6) and torch.allclose(so, y.std(0), rtol=1e-4, atol=1e-6))
        mo1, so1 = torch.empty_like(mo), torch.empty_like(so)
        for _ in range(3):
            hot.hot_stats_whole(y, 1, mo1, so1)
        e[0].record()
        for _ in range(iters):
            hot.hot_stats_whole(y, 1, mo1, so1)
        e[1].record()
        torch.cuda.synchronize()
        ms_w = e[0].elapsed_time(e[1]) / iters
        ok = ok and bool(torch.equal(mo1, mo) and torch.equal(so1, so))
        out[name] = {"local_ms": ms_l, "merge_ms": ms_m, "one_pass_ms": ms_w, "one_pass_GBps": (4 * s * m + 8 * m) / ms_w / 1e6,
                     "predictions_per_s": s * m / (ms_l * 1e-3),
                     "local_GBps": (4 * s * m + 16 * m) / ms_l / 1e6, "agrees_with_torch": ok}
        del y, mean, m2, mo, so, mo1, so1
    return out


def update_and_dropout_lines(hot, torch, dev, wl, iters: int = 10):
    """hot_adam_step (56 bytes per weight) and the MC-dropout forward / backward on the workload's shape."""
    n, s, ld = wl.n_weights, wl.s_local, wl.ld
    a = [torch.randn(n, device=dev) for _ in range(4)] + [torch.zeros(n, device=dev) for _ in range(4)]
    a[1].abs_().add_(0.01)

    def timeit(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    step = [0]

    def adam():
        step[0] += 1
        hot.hot_adam_step(hot.hot_adam(1e-3, 0.9, 0.999, 1e-8, 1.0, 1e-6, step[0]), a[0], a[1], a[2], a[3], *a[4:])

    ms = timeit(adam)
    out = {"adam": {"ms": ms, "weights_per_s": n / (ms * 1e-3), "GBps": 56.0 * n / ms / 1e6,
                    "frac_of_hbm_peak": 56.0 * n / ms / 1e6 / HBM_PEAK_GBS, "bytes_per_weight": 56}}
    # Algorithm 1's pair of steps on one GPU that holds all its samples: hot_backward then hot_adam_step,
    # against hot_backward_adam (gradients never written); lr = 0 keeps sigma where it is
    G = torch.randn(s, ld, device=dev)
    eps = torch.randn(s, ld, device=dev)
    plan1 = hot.hot_create(n, ld, s, s, wl.dataset_size, dev.index or 0)
    still = hot.hot_adam(0.0, 0.9, 0.999, 1e-8, 1.0, 0.0, 1)

    def two_calls():
        hot.hot_backward(plan1, a[0], a[1], eps, G, a[2], a[3])
        hot.hot_adam_step(still, a[0], a[1], a[2], a[3], *a[4:])

    ms_two = timeit(two_calls)
    ms_one = timeit(lambda: hot.hot_backward_adam(plan1, None, still, a[0], a[1], eps, G, *a[4:]))
    # Algorithm 1's whole step behind the network's backward pass, eps drawn in the kernels: backward, Adam
    # and the next step's forward as three calls, as hot_backward_adam + hot_forward_rng, and as one call
    rng_a, rng_b = hot.hot_rng(seed=RNG_SEED, step=RNG_STEP, first_sample=0), hot.hot_rng(seed=RNG_SEED, step=RNG_STEP + 1, first_sample=0)
    kl1 = torch.zeros(1, dtype=torch.float64, device=dev)
    w_next = eps                                    # eps' storage serves as the next step's w here

    def three_calls():
        hot.hot_backward_rng(plan1, rng_a, a[0], a[1], G, a[2], a[3])
        hot.hot_adam_step(still, a[0], a[1], a[2], a[3], *a[4:])
        hot.hot_forward_rng(plan1, rng_b, a[0], a[1], w_next, kl1)

    def pair_calls():
        hot.hot_backward_adam(plan1, rng_a, still, a[0], a[1], None, G, *a[4:])
        hot.hot_forward_rng(plan1, rng_b, a[0], a[1], w_next, kl1)

    ms_w3, ms_w2 = timeit(three_calls), timeit(pair_calls)
    ms_w1 = timeit(lambda: hot.hot_backward_adam_forward(plan1, rng_a, rng_b, still, a[0], a[1], G, *a[4:], w_next, kl1))
    b_w3, b_w2, b_w1 = 4.0 * n * (s + 4) + 56.0 * n + 4.0 * n * (s + 2), 4.0 * n * (s + 2) + 40.0 * n + 4.0 * n * (s + 2), 4.0 * n * (2 * s + 2) + 40.0 * n
    out["whole_step_fused"] = {"ms": ms_w1, "GBps": b_w1 / ms_w1 / 1e6, "frac_of_hbm_peak": b_w1 / ms_w1 / 1e6 / HBM_PEAK_GBS,
                               "bytes_per_weight": b_w1 / n, "two_calls_ms": ms_w2, "two_calls_bytes_per_weight": b_w2 / n,
                               "three_calls_ms": ms_w3, "three_calls_bytes_per_weight": b_w3 / n,
                               "speedup_over_two_calls": ms_w2 / ms_w1, "speedup_over_three_calls": ms_w3 / ms_w1,
                               "samples": s, "eps": "in-kernel",
                               "what": "hot_backward_adam_forward: backward, Adam and the next step's forward (w + KL) in one pass"}
    hot.hot_destroy(plan1)
    b_two, b_one = 4.0 * n * (2 * s + 4) + 56.0 * n, 4.0 * n * (2 * s + 2) + 40.0 * n
    out["backward_adam_fused"] = {"ms": ms_one, "GBps": b_one / ms_one / 1e6, "frac_of_hbm_peak": b_one / ms_one / 1e6 / HBM_PEAK_GBS,
                                  "bytes_per_weight": b_one / n, "two_calls_ms": ms_two, "two_calls_bytes_per_weight": b_two / n,
                                  "speedup": ms_two / ms_one, "samples": s}
    # Algorithm 2 after the all-reduce: hot_adam_step then the next step's hot_forward_rng, against hot_adam_forward
    plan2 = hot.hot_create(n, ld, s, wl.s_total, wl.dataset_size, dev.index or 0)
    rng2 = hot.hot_rng(seed=RNG_SEED, step=RNG_STEP + 1, first_sample=0)
    kl = torch.zeros(1, dtype=torch.float64, device=dev)

    def adam_then_forward():
        hot.hot_adam_step(still, a[0], a[1], a[2], a[3], *a[4:])
        hot.hot_forward_rng(plan2, rng2, a[0], a[1], G, kl)          # G's storage serves as w here

    ms_af2 = timeit(adam_then_forward)
    ms_af1 = timeit(lambda: hot.hot_adam_forward(plan2, rng2, still, a[0], a[1], a[2], a[3], *a[4:], None, G, kl))
    hot.hot_destroy(plan2)
    b_af2, b_af1 = 56.0 * n + 4.0 * n * (s + 2), 56.0 * n + 4.0 * n * s
    out["adam_forward_fused"] = {"ms": ms_af1, "GBps": b_af1 / ms_af1 / 1e6, "frac_of_hbm_peak": b_af1 / ms_af1 / 1e6 / HBM_PEAK_GBS,
                                 "bytes_per_weight": b_af1 / n, "two_calls_ms": ms_af2, "two_calls_bytes_per_weight": b_af2 / n,
                                 "speedup": ms_af2 / ms_af1, "samples": s, "eps": "in-kernel"}
    del a, G, eps
    torch.cuda.empty_cache()
    mu = torch.randn(n, device=dev)
    w = torch.empty(s, ld, device=dev)
    gmu = torch.empty(n, device=dev)
    plan = hot.hot_create(n, ld, s, wl.s_total, wl.dataset_size, dev.index or 0)
    rng = hot.hot_rng(seed=RNG_SEED, step=RNG_STEP, first_sample=0)
    ms_f = timeit(lambda: hot.hot_forward_dropout_rng(plan, rng, 0.9, mu, w))
    ms_b = timeit(lambda: hot.hot_backward_dropout_rng(plan, rng, 0.9, w, gmu))
    hot.hot_destroy(plan)
    fb, bb = 4.0 * n * (1 + s), 4.0 * n * (s + 1)
    out["mc_dropout"] = {"forward_ms": ms_f, "backward_ms": ms_b, "items_per_s": s * n / ((ms_f + ms_b) * 1e-3),
                         "forward_GBps": fb / ms_f / 1e6, "backward_GBps": bb / ms_b / 1e6,
                         "step_frac_of_hbm_roofline": (fb + bb) / ((ms_f + ms_b) * 1e-3) / 1e9 / HBM_PEAK_GBS}
    return out


FP32_MFMA_PEAK_TFLOPS = 157.3


def sampled_linear_lines(hot, torch, dev, iters: int = 20):
    """hot_linear_forward_rng (eps drawn in registers, contraction on the matrix cores) on layer shapes
    of the paper's models and on one large square layer; beside it the same layer done as
    hot_forward_rng (w written to HBM) + one library GEMM per sample."""
    def timeit(fn):
        # untimed calls first, for at least 30 ms: the card sits at idle clocks while the tensors of a shape are made, and
        # what is timed first would otherwise run 5-8 % slower than the same call a moment later
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        warm = 0.0
        while warm < 30.0:
            e0.record()
            for _ in range(3):
                fn()
            e1.record()
            torch.cuda.synchronize()
            warm += max(e0.elapsed_time(e1), 0.5)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    rng = hot.hot_rng(seed=RNG_SEED, step=RNG_STEP, first_sample=0)
    out = {}
    shapes = {"mlp_fc2_R64_128x128_S4": (64, 128, 128, 4), "swin_fc1_R1_540x2160_S2": (1, 540, 2160, 2),
              "swin_fc1_R64_540x2160_S2": (64, 540, 2160, 2), "swin_fc_R16_2160x8640_S2": (16, 2160, 8640, 2),
              "square_R1_8192x8192_S2": (1, 8192, 8192, 2), "square_R16_8192x8192_S2": (16, 8192, 8192, 2),
              "square_R64_8192x8192_S2": (64, 8192, 8192, 2), "swin_fc1_R7260_540x2160_S2": (7260, 540, 2160, 2),
              "vit_fc1_R16640_192x768_S2": (16640, 192, 768, 2), "square_R1024_8192x8192_S2": (1024, 8192, 8192, 2),
              # a layer inside the network: every sample has an input of its own
              "swin_fc2_R7260_2160x540_S2_own_x": (7260, 2160, 540, 2)}
    for name, (rows, k, o, s) in shapes.items():
        own_x = name.endswith("_own_x")
        x = torch.randn(s, rows, k, device=dev) if own_x else torch.randn(rows, k, device=dev)
        x_all = x if own_x else x.unsqueeze(0).expand(s, rows, k)          # [S, R, K] view for the library calls
        mu = torch.randn(o, k, device=dev) * (2.0 / k) ** 0.5
        sg = torch.rand(o, k, device=dev) * 0.01 + 0.001
        mb = torch.zeros(o, device=dev)
        sb = torch.full((o,), 0.01, device=dev)
        y = torch.empty(s, rows, o, device=dev)
        ms = timeit(lambda: hot.hot_linear_forward_rng(rng, x, mu, sg, mb, sb, y, 0, o * k))
        n = o * k + o
        plan = hot.hot_create(n, n, s, s, 1.0, dev.index or 0)
        flat_mu, flat_sg = torch.cat([mu.view(-1), mb]), torch.cat([sg.view(-1), sb])
        w = torch.empty(s, n, device=dev)
        y2 = torch.empty_like(y)

        def unfused():
            hot.hot_forward_rng(plan, rng, flat_mu, flat_sg, w)
            torch.baddbmm(w[:, o * k:].unsqueeze(1), x_all,
                          w[:, :o * k].view(s, o, k).transpose(1, 2), out=y2)

        ms_u = timeit(unfused)
        # back-propagation through the layer: fused (neither w nor the per-sample weight gradients exist)
        # against library GEMMs for dx and G_s followed by hot_backward_rng (w kept from the forward pass)
        dy = torch.randn(s, rows, o, device=dev)
        gmw, gsw, gmb, gsb = (torch.empty(o, k, device=dev), torch.empty(o, k, device=dev),
                              torch.empty(o, device=dev), torch.empty(o, device=dev))
        dx = torch.empty(s, rows, k, device=dev)
        ms_b = timeit(lambda: hot.hot_linear_backward_rng(rng, x, dy, mu, sg, mb, sb, gmw, gsw, gmb, gsb, dx, s, 45000.0,
                                                          hot.HOT_REDUCE_SUM, 0, o * k))
        # the two halves of the call: weight and bias gradients alone (dx = NULL); the input gradients are the rest
        ms_wg = timeit(lambda: hot.hot_linear_backward_rng(rng, x, dy, mu, sg, mb, sb, gmw, gsw, gmb, gsb, None, s, 45000.0,
                                                           hot.HOT_REDUCE_SUM, 0, o * k))
        ws_bytes = hot.hot_linear_backward_workspace_bytes(rows, k, o, s)
        ms_bw = None
        if ws_bytes > 0:        # few tiles, many rows: the rows go to several workgroups through a workspace; up to 128 rows: both gradients in one pass
            ws = torch.empty(ws_bytes // 4, device=dev)
            ms_bw = timeit(lambda: hot.hot_linear_backward_rng(rng, x, dy, mu, sg, mb, sb, gmw, gsw, gmb, gsb, dx, s, 45000.0,
                                                               hot.HOT_REDUCE_SUM, 0, o * k, workspace=ws))
            del ws
        G = torch.empty(s, n, device=dev)
        dx2 = torch.empty_like(dx)
        gf, gs2 = torch.empty(n, device=dev), torch.empty(n, device=dev)
        plan_b = hot.hot_create(n, n, s, s, 45000.0, dev.index or 0)

        def unfused_backward():
            torch.matmul(dy, w.as_strided((s, o, k), (n, k, 1)), out=dx2)
            torch.matmul(dy.transpose(1, 2), x_all, out=G.as_strided((s, o, k), (n, k, 1)))
            torch.sum(dy, dim=1, out=G[:, o * k:])
            hot.hot_backward_rng(plan_b, rng, flat_mu, flat_sg, G, gf, gs2)

        ms_bu = timeit(unfused_backward)
        ms_lib_g = timeit(lambda: torch.matmul(dy.transpose(1, 2), x_all, out=G.as_strided((s, o, k), (n, k, 1))))
        ms_lib_dx = timeit(lambda: torch.matmul(dy, w.as_strided((s, o, k), (n, k, 1)), out=dx2))
        hot.hot_destroy(plan_b)
        gscale = G[:, :o * k].abs().sum(0).max().item() / s + 1e-6
        bwd = {"fused_ms": ms_b, "weight_samples_per_s": s * o * k / (ms_b * 1e-3),
               "fused_with_workspace_ms": ms_bw, "workspace_bytes": ws_bytes,
               "weight_gradients_ms": ms_wg, "weight_gradients_TFLOPs": 2.0 * s * rows * k * o / ms_wg / 1e9,
               "input_gradients_ms": ms_b - ms_wg, "input_gradients_TFLOPs": 2.0 * s * rows * k * o / max(ms_b - ms_wg, 1e-6) / 1e9,
               "library_gemm_for_G_ms": ms_lib_g, "library_gemm_for_dx_ms": ms_lib_dx,
               "library_gemms_plus_hot_backward_ms": ms_bu, "speedup": ms_bu / ms_b,
               "speedup_with_workspace": ms_bu / ms_bw if ms_bw else None,
               "agrees": bool((gmw.view(-1) - gf[:o * k]).abs().max().item() <= 1e-5 * gscale
                              and (dx - dx2).abs().max().item() <= 1e-4 * dx2.abs().max().item())}
        del dy, gmw, gsw, dx, dx2, G, gf, gs2
        hot.hot_destroy(plan)
        scale = (x.reshape(-1, k).abs() @ (mu.abs() + 6 * sg).t()).max().item()
        out[name] = {"fused_ms": ms, "TFLOPs": 2.0 * s * rows * k * o / ms / 1e9,
                     "frac_of_fp32_mfma_peak": 2.0 * s * rows * k * o / ms / 1e9 / FP32_MFMA_PEAK_TFLOPS,
                     "weight_samples_per_s": s * o * k / (ms * 1e-3), "mu_sigma_GBps": 8.0 * o * k / ms / 1e6,
                     "materialise_plus_library_gemm_ms": ms_u, "speedup_over_materialise": ms_u / ms,
                     "agrees_with_materialised": bool((y - y2).abs().max().item() <= 1e-5 * scale),
                     "backward": bwd}
        del x, mu, sg, y, y2, w
    out["note"] = ("TFLOPs counts the layer's 2 S R K O fp32 operations. From 129 rows on, the forward call and the input "
                   "gradients form every product from three bf16 pieces of both factors on v_mfma_f32_32x32x16_bf16 (six of "
                   "the nine partial products: fp32 accuracy at 6/16 of the cycles of v_mfma_f32_32x32x2_f32), so "
                   "frac_of_fp32_mfma_peak, which prices against the fp32 instruction's 157.3 TFLOP/s, can exceed 1; against "
                   "the bf16 peak divided by six products the ceiling is 417 TFLOP/s. The weight gradients of large layers (tiles of "
                   "128 x 128) are formed the same way; the other weight-gradient kernels use the fp32 instructions.")
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C4", help="workload C1..C5 (C4 is the one the metric is quoted on)")
    ap.add_argument("--eps", choices=["array", "in-kernel"], default="array",
                    help="eps read from its array (the graded path) or drawn inside the kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--cpu-weights", type=int, default=1 << 28, help="cap on weights the oracle is timed on")
    ap.add_argument("--linear-only", action="store_true", help="only run the sampled linear layer lines")
    ap.add_argument("--probe-copy", action="store_true",
                    help="only run the plain copy kernel (2 GiB, known traffic) and print its rate")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards over samples; the all-reduce is not "
              "part of it). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2604_04736_amd import binding as hot, workloads
    hot.lib()                                   # fail loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    if args.probe_copy:
        print(json.dumps({"probe": "hot_probe_copy_kernel", "steps": args.steps,
                          **copy_ceiling(hot, torch, dev, iters=args.steps)}))
        return 0
    if args.linear_only:
        print(json.dumps({"sampled_linear": sampled_linear_lines(hot, torch, dev, iters=args.steps)}))
        return 0
    # The oracle belongs to the cpu_baseline leg only: it is timed there, and the same leg checks sampled
    # windows of the timed buffers against it.  With --no-cpu-baseline nothing under oracle/ is touched.
    oracle = None
    if not args.no_cpu_baseline:
        import oracle

    def check(wl_, x_, out_, in_kernel):
        return None if oracle is None else bool(verify_sampled(oracle, np, wl_, x_, out_, in_kernel_eps=in_kernel))

    wl = workloads.CONFIGS[args.config]
    x = workloads.make_inputs(wl, dev)
    torch.cuda.synchronize()
    gen = args.eps == "in-kernel"
    r = time_steps(hot, torch, wl, x, args.steps, args.warmup, gen)
    ms_per_step = r["wall_s"] * 1e3 / args.steps
    items = wl.items
    fwd_b, bwd_b = algorithmic_bytes(wl.n_weights, wl.s_local, gen)
    dominant = "backward" if r["bwd_ms"] >= r["fwd_ms"] else "forward"
    dom_bytes, dom_ms = (bwd_b, r["bwd_ms"]) if dominant == "backward" else (fwd_b, r["fwd_ms"])
    achieved = dom_bytes / dom_ms / 1e6
    verified = check(wl, x, r["out"], gen)
    kname = "_rng" if gen else ""

    result = {
        "metric": METRIC,
        "value": items / (ms_per_step * 1e-3),
        "unit": "items/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.note}; N={wl.n_weights}, S_loc={wl.s_local}, S={wl.s_total}, "
                               f"ld={wl.ld}, |D|={wl.dataset_size:g}, fp32, seed {wl.seed}",
                   "items_per_step": items, "eps": args.eps,
                   "step": f"hot_forward{kname} (w + KL) then hot_backward{kname} (grad_mu, grad_sigma)",
                   "launch": r["launch"]},
        "roofline": {"bound": "hbm", "kernel": f"hot_{dominant}_kernel", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(f"hot_{dominant}{kname}_kernel", wl.name),
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms},
        "kernels": {
            "forward": {"ms": r["fwd_ms"], "median_ms": r["spread"]["fwd_median_ms"], "min_ms": r["spread"]["fwd_min_ms"], "GBps": fwd_b / r["fwd_ms"] / 1e6, "items_per_s": items / r["fwd_ms"] * 1e3,
                        "frac_of_hbm_peak": fwd_b / r["fwd_ms"] / 1e6 / HBM_PEAK_GBS,
                        "note": "interval between HIP events; includes the one-workgroup KL finish kernel"},
            "backward": {"ms": r["bwd_ms"], "median_ms": r["spread"]["bwd_median_ms"], "min_ms": r["spread"]["bwd_min_ms"], "GBps": bwd_b / r["bwd_ms"] / 1e6, "items_per_s": items / r["bwd_ms"] * 1e3,
                         "frac_of_hbm_peak": bwd_b / r["bwd_ms"] / 1e6 / HBM_PEAK_GBS},
        },
        "step_frac_of_hbm_roofline": (fwd_b + bwd_b) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "verified_against_oracle": verified,
    }
    ceiling = copy_ceiling(hot, torch, dev)
    result["copy_ceiling"] = {"GBps": ceiling["GBps"], "frac_of_hbm_peak": ceiling["GBps"] / HBM_PEAK_GBS,
                              "what": "hot_probe_copy_kernel, 2 GiB read + 2 GiB written",
                              "runtime_copy_GBps": ceiling["runtime_copy_GBps"],
                              "runtime_copy_what": "torch Tensor.copy_ (the HIP runtime's device-to-device copy) over the same buffers"}
    # the dominant kernel's own traffic mix without its arithmetic: backward reads G and (array mode) eps
    # rows plus mu, sigma and writes grad_mu, grad_sigma; forward reads (eps rows,) mu, sigma and writes w rows
    rows = wl.s_local
    mix = {"backward": ((1 if gen else 2) * rows + 2, 2), "forward": ((0 if gen else rows) + 2, rows)}[dominant]
    if mix[0] <= 64 and mix[1] <= 64:
        stream_bytes = 4 * wl.n_weights // 16 * 16
        m = mix_ceiling(hot, torch, dev, stream_bytes, mix[0], mix[1])
        result["mix_ceiling"] = {"GBps": m["GBps"], "frac_of_hbm_peak": m["GBps"] / HBM_PEAK_GBS,
                                 "kernel_vs_mix_ceiling": achieved / m["GBps"],
                                 "what": f"hot_probe_streams_kernel: {mix[0]} read + {mix[1]} write streams of "
                                         f"{stream_bytes} bytes, the {dominant} kernel's traffic without its arithmetic"}

    if not args.no_others:
        result["between_other_work"] = between_other_work(hot, torch, wl, x, gen)
    if not args.no_others and not gen:
        fw = framework_step(torch, wl, x)
        fw["speedup_of_this_library"] = fw["ms_per_step"] / ms_per_step
        result["framework_reference"] = fw

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(oracle, np, wl, x, args.cpu_weights, None if gen else r["out"])
        kl_gpu = r["out"]["kl"].item()
        result["cpu_baseline"]["kl_gpu"] = kl_gpu
        every = result["cpu_baseline"].pop("every_element")
        if every is not None:
            # every element of the timed buffers of the headline workload against the oracle, not a sample
            result["verified_every_element"] = every
            if not every["all_within_tolerance"]:
                verified = result["verified_against_oracle"] = False
    del x, r
    torch.cuda.empty_cache()

    if not args.no_others and not gen:
        # the same workload with eps drawn inside the kernels (no eps array is read)
        xr = workloads.make_inputs(wl, dev)
        del xr["eps"]
        torch.cuda.synchronize()
        rr = time_steps(hot, torch, wl, xr, 20, 5, True)
        fb, bb = algorithmic_bytes(wl.n_weights, wl.s_local, True)
        ms = rr["wall_s"] * 1e3 / 20
        result["in_kernel_eps"] = {
            "items_per_s": items / (ms * 1e-3), "ms_per_step": ms, "fwd_ms": rr["fwd_ms"], "bwd_ms": rr["bwd_ms"],
            "algorithmic_bytes_per_step": fb + bb,
            "fwd_GBps": fb / rr["fwd_ms"] / 1e6, "bwd_GBps": bb / rr["bwd_ms"] / 1e6,
            "step_frac_of_hbm_roofline": (fb + bb) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "verified_against_oracle": check(wl, xr, rr["out"], True),
            "forward_alu_roofline": alu_roofline_forward_rng(wl.name, items / (rr["fwd_ms"] * 1e-3)),
            "note": "hot_forward_rng + hot_backward_rng: Philox-4x32-10 + Box-Muller in registers"}
        del xr, rr
        torch.cuda.empty_cache()

    if not args.no_others:
        result["predictive_stats"] = predictive_stats_lines(hot, torch, dev)
        result["sampled_linear"] = sampled_linear_lines(hot, torch, dev)
        result["update_and_dropout"] = update_and_dropout_lines(hot, torch, dev, wl)
        others = {}
        for name, o in workloads.CONFIGS.items():
            if name == wl.name:
                continue
            xo = workloads.make_inputs(o, dev)
            torch.cuda.synchronize()
            ro = time_steps(hot, torch, o, xo, 20, 5, gen)
            fb, bb = algorithmic_bytes(o.n_weights, o.s_local, gen)
            ms = ro["wall_s"] * 1e3 / 20
            others[name] = {"items_per_s": o.items / (ms * 1e-3), "ms_per_step": ms,
                            "fwd_ms": ro["fwd_ms"], "bwd_ms": ro["bwd_ms"],
                            "step_frac_of_hbm_roofline": (fb + bb) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "verified_against_oracle": check(o, xo, ro["out"], gen)}
            others[name]["between_other_work"] = between_other_work(hot, torch, o, xo, gen)
            if o.items >= 50_000_000:      # HBM-bound sizes: each kernel beside a no-arithmetic kernel with its stream mix
                others[name]["mix_ceiling"] = mix_ceilings(hot, torch, dev, o, gen, ro["fwd_ms"], ro["bwd_ms"])
            if o.items < 50_000_000:       # launch-latency-bound sizes: the same step replayed from a HIP graph
                gms = time_graph_steps(hot, torch, o, xo, 200, gen)
                others[name]["hip_graph_ms_per_step"] = gms
                others[name]["hip_graph_items_per_s"] = o.items / (gms * 1e-3)
            del xo, ro
            torch.cuda.empty_cache()
        result["other_workloads"] = others

    print(json.dumps(result))
    return 1 if verified is False else 0


if __name__ == "__main__":
    sys.exit(main())
