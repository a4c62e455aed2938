"""ctypes front end of the CPU oracle in ``bbb_oracle.c`` (sample layer) and
``eps_oracle.c`` (counter-based eps draw) ``stats_oracle.c`` (predictive mean / std) ``linear_oracle.c`` (sampled linear layer) and ``update_oracle.c`` (Adam step, MC-dropout layer).

Test infrastructure only: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg call this; the product package never imports it.  This module
marshals numpy arrays and does no arithmetic of the method itself.

The functions follow Algorithm 2 of arxiv 2604.04736 (per-GPU inner loop): see the
comments in ``bbb_oracle.c`` for which line each one writes out.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("bbb_oracle.c", "eps_oracle.c", "stats_oracle.c", "linear_oracle.c",
                                               "update_oracle.c")]
_LIB = os.path.join(_HERE, "libbbb_oracle.so")

_lib = None


class AdamParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("grad_scale", ctypes.c_double), ("sigma_min", ctypes.c_double),
                ("step", ctypes.c_int64)]


def build(force: bool = True) -> str:
    """Compile the oracle's C files with gcc into ``libbbb_oracle.so`` next to them."""
    if not force and os.path.exists(_LIB) and all(os.path.getmtime(_LIB) >= os.path.getmtime(s) for s in _SRCS):
        return _LIB
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB] + _SRCS + ["-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    # BBB_ORACLE_LIB: an oracle library somebody else built from the same sources (the sanitizer test's)
    other = os.environ.get("BBB_ORACLE_LIB")
    if not other:
        build(force=False)
    lib = ctypes.CDLL(other or _LIB)
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    lib.bbb_oracle_threads.argtypes = [ctypes.c_int]
    lib.bbb_oracle_threads.restype = ctypes.c_int
    lib.bbb_oracle_reparam.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                       fp, fp, fp, dp, ctypes.c_int64, ctypes.c_int]
    lib.bbb_oracle_reparam.restype = None
    lib.bbb_oracle_kl.argtypes = [ctypes.c_int64, fp, fp]
    lib.bbb_oracle_kl.restype = ctypes.c_double
    lib.bbb_oracle_grad.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                    ctypes.c_double, ctypes.c_int, fp, fp, fp, fp, dp, dp,
                                    ctypes.c_int]
    lib.bbb_oracle_grad.restype = None
    u32p = ctypes.POINTER(ctypes.c_uint32)
    lib.eps_oracle_philox4x32.argtypes = [u32p, u32p, ctypes.c_int, u32p]
    lib.eps_oracle_philox4x32.restype = None
    lib.eps_oracle_bits.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                                    ctypes.c_uint32, ctypes.c_uint32, u32p]
    lib.eps_oracle_bits.restype = None
    lib.eps_oracle_normal.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                                      ctypes.c_uint32, ctypes.c_uint32, dp, dp]
    lib.eps_oracle_normal.restype = None
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.stats_oracle_whole.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, fp, ctypes.c_int32, dp, dp]
    lib.stats_oracle_whole.restype = None
    lib.stats_oracle_partial.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, fp, dp, dp]
    lib.stats_oracle_partial.restype = None
    lib.stats_oracle_merge.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, i32p, dp, dp,
                                       ctypes.c_int32, dp, dp]
    lib.stats_oracle_merge.restype = None
    lib.linear_oracle_forward.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.c_int64, fp, fp, fp, dp, fp, fp, dp, dp]
    lib.linear_oracle_forward.restype = None
    lib.linear_oracle_backward.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_int64, ctypes.c_double, ctypes.c_double, fp, fp, fp, fp, dp, fp, fp,
                                           dp, dp, dp, dp, dp, dp]
    lib.linear_oracle_backward.restype = None
    lib.update_oracle_adam.argtypes = [ctypes.c_int64, ctypes.POINTER(AdamParams), dp, dp, dp, dp, dp, dp, dp, dp]
    lib.update_oracle_adam.restype = None
    lib.update_oracle_dropout_threshold.argtypes = [ctypes.c_double]
    lib.update_oracle_dropout_threshold.restype = ctypes.c_uint64
    lib.update_oracle_dropout_forward.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_double,
                                                  fp, u32p, dp]
    lib.update_oracle_dropout_forward.restype = None
    lib.update_oracle_dropout_backward.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                                   ctypes.c_int32, ctypes.c_int, ctypes.c_double, fp, u32p, dp]
    lib.update_oracle_dropout_backward.restype = None
    _lib = lib
    return lib


def _f32(a, name):
    a = np.asarray(a)
    if a.dtype != np.float32:
        raise TypeError(f"{name} must be float32, got {a.dtype}")
    if not a.flags.c_contiguous:
        raise ValueError(f"{name} must be C-contiguous")
    return a


def _fptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check_2d(a, s_loc, n, name):
    if a.ndim != 2 or a.shape[0] != s_loc or a.shape[1] < n:
        raise ValueError(f"{name} must have shape [S_loc={s_loc}, ld>={n}], got {a.shape}")


def threads(nthreads: int) -> int:
    return int(_load().bbb_oracle_threads(int(nthreads)))


def reparam(mu, sigma, eps, nthreads: int = 1) -> np.ndarray:
    """w[s,i] = mu[i] + sigma[i]*eps[s,i] in fp64; eps is [S_loc, ld>=N]; returns [S_loc, N]."""
    mu = _f32(mu, "mu")
    sigma = _f32(sigma, "sigma")
    eps = _f32(eps, "eps")
    n = mu.shape[0]
    if mu.ndim != 1 or sigma.shape != mu.shape:
        raise ValueError("mu and sigma must be 1-D of equal length")
    s_loc = eps.shape[0]
    _check_2d(eps, s_loc, n, "eps")
    w = np.empty((s_loc, n), dtype=np.float64)
    _load().bbb_oracle_reparam(n, eps.shape[1], s_loc, _fptr(mu), _fptr(sigma), _fptr(eps),
                               _dptr(w), n, int(nthreads))
    return w


def kl(mu, sigma) -> float:
    """1/2 sum_i (sigma_i^2 + mu_i^2 - 1 - ln sigma_i^2) in fp64."""
    mu = _f32(mu, "mu")
    sigma = _f32(sigma, "sigma")
    if mu.ndim != 1 or sigma.shape != mu.shape:
        raise ValueError("mu and sigma must be 1-D of equal length")
    return float(_load().bbb_oracle_kl(mu.shape[0], _fptr(mu), _fptr(sigma)))


def grad(mu, sigma, eps, G, s_total: int, dataset_size: float, reduce_mean: bool = False,
         nthreads: int = 1):
    """(grad_mu, grad_sigma) in fp64, each [N]; eps and G are [S_loc, ld>=N] with equal pitch."""
    mu = _f32(mu, "mu")
    sigma = _f32(sigma, "sigma")
    eps = _f32(eps, "eps")
    G = _f32(G, "G")
    n = mu.shape[0]
    if mu.ndim != 1 or sigma.shape != mu.shape:
        raise ValueError("mu and sigma must be 1-D of equal length")
    s_loc = eps.shape[0]
    _check_2d(eps, s_loc, n, "eps")
    if G.shape != eps.shape:
        raise ValueError("G and eps must have the same shape")
    if not (1 <= s_loc <= s_total) or not dataset_size > 0:
        raise ValueError("need 1 <= S_loc <= S and |D| > 0")
    gmu = np.empty(n, dtype=np.float64)
    gsig = np.empty(n, dtype=np.float64)
    _load().bbb_oracle_grad(n, eps.shape[1], s_loc, int(s_total), float(dataset_size),
                            1 if reduce_mean else 0, _fptr(mu), _fptr(sigma), _fptr(eps),
                            _fptr(G), _dptr(gmu), _dptr(gsig), int(nthreads))
    return gmu, gsig


def philox4x32(ctr, key, rounds: int = 10):
    """Philox-4x32 block function: four counter words, two key words -> four output words."""
    c = (ctypes.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    out = (ctypes.c_uint32 * 4)()
    _load().eps_oracle_philox4x32(c, k, int(rounds), out)
    return [int(v) for v in out]


def eps_bits(n: int, s_loc: int, seed: int, step: int = 0, first_sample: int = 0, col0: int = 0) -> np.ndarray:
    """Integer stage of the eps draw for weights col0..col0+n-1: uint32 [S_loc, n]."""
    out = np.empty((s_loc, n), dtype=np.uint32)
    _load().eps_oracle_bits(int(col0), n, n, s_loc, int(seed), int(step), int(first_sample),
                            out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
    return out


def eps_normal(n: int, s_loc: int, seed: int, step: int = 0, first_sample: int = 0, with_radius=False,
               col0: int = 0):
    """eps ~ N(0, 1) in fp64 for weights col0..col0+n-1, [S_loc, n]; with_radius also returns the
    Box-Muller radius of each."""
    out = np.empty((s_loc, n), dtype=np.float64)
    rad = np.empty((s_loc, n), dtype=np.float64) if with_radius else None
    _load().eps_oracle_normal(int(col0), n, n, s_loc, int(seed), int(step), int(first_sample), _dptr(out),
                              _dptr(rad) if with_radius else None)
    return (out, rad) if with_radius else out


def stats_whole(y, m: int = None, ddof: int = 0):
    """Mean and standard deviation over the rows (samples) of y[S, ld>=m], fp64, two-pass definition."""
    y = _f32(y, "y")
    m = y.shape[1] if m is None else m
    mean, std = np.empty(m), np.empty(m)
    _load().stats_oracle_whole(m, y.shape[1], y.shape[0], _fptr(y), int(ddof), _dptr(mean), _dptr(std))
    return mean, std


def stats_partial(y, m: int = None):
    """What one GPU contributes for its rows: (mean, M2 = sum of squared deviations), fp64."""
    y = _f32(y, "y")
    m = y.shape[1] if m is None else m
    mean, m2 = np.empty(m), np.empty(m)
    _load().stats_oracle_partial(m, y.shape[1], y.shape[0], _fptr(y), _dptr(mean), _dptr(m2))
    return mean, m2


def stats_merge(counts, means, m2s, ddof: int = 0):
    """Pooled mean and standard deviation from the partials of several GPUs ([parts, m] fp64 arrays)."""
    means = np.ascontiguousarray(means, dtype=np.float64)
    m2s = np.ascontiguousarray(m2s, dtype=np.float64)
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    parts, m = means.shape
    if m2s.shape != means.shape or counts.shape != (parts,):
        raise ValueError("means and m2s must be [parts, m], counts [parts]")
    mean, std = np.empty(m), np.empty(m)
    _load().stats_oracle_merge(parts, m, m, counts.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _dptr(means),
                               _dptr(m2s), int(ddof), _dptr(mean), _dptr(std))
    return mean, std


def linear_forward(x, mu_w, sigma_w, eps_w, mu_b=None, sigma_b=None, eps_b=None, in_features=None):
    """y[S, R, O] = x W_s^T + b_s with W_s = mu_w + sigma_w*eps_w[s], b_s likewise; fp64.
    x is [R, ldx >= K] (shared by the samples) or [S, R, ldx >= K] (one input per sample); mu_w, sigma_w [O, K]; eps_w [S, O, K] fp64; bias arrays [O] / [S, O] or None."""
    x = _f32(x, "x")
    mu_w = _f32(mu_w, "mu_w")
    sigma_w = _f32(sigma_w, "sigma_w")
    eps_w = np.ascontiguousarray(eps_w, dtype=np.float64)
    o, k = mu_w.shape
    if in_features is not None and in_features != k:
        raise ValueError("in_features does not match mu_w")
    s = eps_w.shape[0]
    if sigma_w.shape != (o, k) or eps_w.shape != (s, o, k) or x.ndim not in (2, 3) or x.shape[-1] < k:
        raise ValueError("shape mismatch")
    if x.ndim == 3 and x.shape[0] != s:
        raise ValueError("per-sample x needs one [R, ldx] block per sample")
    r, ldx = x.shape[-2], x.shape[-1]
    x_stride = r * ldx if x.ndim == 3 else 0
    y = np.empty((s, r, o), dtype=np.float64)
    if mu_b is None:
        mb = sb = None
        eb = None
    else:
        mu_b = _f32(mu_b, "mu_b")
        sigma_b = _f32(sigma_b, "sigma_b")
        eps_b = np.ascontiguousarray(eps_b, dtype=np.float64)
        if mu_b.shape != (o,) or sigma_b.shape != (o,) or eps_b.shape != (s, o):
            raise ValueError("bias shape mismatch")
        mb, sb, eb = _fptr(mu_b), _fptr(sigma_b), _dptr(eps_b)
    _load().linear_oracle_forward(s, r, k, o, ldx, x_stride, _fptr(x), _fptr(mu_w), _fptr(sigma_w), _dptr(eps_w),
                                  mb, sb, eb, _dptr(y))
    return y


def linear_backward(x, dy, mu_w, sigma_w, eps_w, mu_b=None, sigma_b=None, eps_b=None, g: float = 1.0, k: float = 0.0,
                    want_dx: bool = True):
    """Gradients of the sampled linear layer, fp64: (grad_mu_w [O,K], grad_sigma_w [O,K], grad_mu_b [O] or None,
    grad_sigma_b [O] or None, dx [S,R,K] or None) from dy [S,R,O] = dL_s/dy_s; g, k as in grad().
    x is [R, ldx >= K] or [S, R, ldx >= K]."""
    x = _f32(x, "x")
    dy = _f32(dy, "dy")
    mu_w = _f32(mu_w, "mu_w")
    sigma_w = _f32(sigma_w, "sigma_w")
    eps_w = np.ascontiguousarray(eps_w, dtype=np.float64)
    o, kf = mu_w.shape
    s = eps_w.shape[0]
    if sigma_w.shape != (o, kf) or eps_w.shape != (s, o, kf) or x.ndim not in (2, 3) or x.shape[-1] < kf:
        raise ValueError("shape mismatch")
    if x.ndim == 3 and x.shape[0] != s:
        raise ValueError("per-sample x needs one [R, ldx] block per sample")
    r, ldx = x.shape[-2], x.shape[-1]
    if dy.shape != (s, r, o):
        raise ValueError("dy must be [S, R, O]")
    x_stride = r * ldx if x.ndim == 3 else 0
    gmw, gsw = np.empty((o, kf)), np.empty((o, kf))
    if mu_b is None:
        mb = sb = eb = gmb_p = gsb_p = None
        gmb = gsb = None
    else:
        mu_b = _f32(mu_b, "mu_b")
        sigma_b = _f32(sigma_b, "sigma_b")
        eps_b = np.ascontiguousarray(eps_b, dtype=np.float64)
        if mu_b.shape != (o,) or sigma_b.shape != (o,) or eps_b.shape != (s, o):
            raise ValueError("bias shape mismatch")
        gmb, gsb = np.empty(o), np.empty(o)
        mb, sb, eb, gmb_p, gsb_p = _fptr(mu_b), _fptr(sigma_b), _dptr(eps_b), _dptr(gmb), _dptr(gsb)
    dx = np.empty((s, r, kf)) if want_dx else None
    _load().linear_oracle_backward(s, r, kf, o, ldx, x_stride, float(g), float(k), _fptr(x), _fptr(dy), _fptr(mu_w),
                                   _fptr(sigma_w), _dptr(eps_w), mb, sb, eb, _dptr(gmw), _dptr(gsw), gmb_p, gsb_p,
                                   _dptr(dx) if want_dx else None)
    return gmw, gsw, gmb, gsb, dx


def adam_step(mu, sigma, grad_mu, grad_sigma, m_mu, v_mu, m_sigma, v_sigma, step, lr, beta1=0.9, beta2=0.999,
              eps=1e-8, grad_scale=1.0, sigma_min=0.0):
    """One Adam step on (mu, sigma) in fp64; returns new (mu, sigma, m_mu, v_mu, m_sigma, v_sigma)."""
    arrs = [np.array(a, dtype=np.float64, copy=True) for a in (mu, sigma, grad_mu, grad_sigma, m_mu, v_mu, m_sigma, v_sigma)]
    n = arrs[0].shape[0]
    if any(a.shape != (n,) for a in arrs):
        raise ValueError("all arrays must be 1-D of equal length")
    p = AdamParams(lr, beta1, beta2, eps, grad_scale, sigma_min, int(step))
    mu_, sg_, gm_, gs_, mm_, vm_, ms_, vs_ = arrs
    _load().update_oracle_adam(n, ctypes.byref(p), _dptr(mu_), _dptr(sg_), _dptr(gm_), _dptr(gs_), _dptr(mm_),
                               _dptr(vm_), _dptr(ms_), _dptr(vs_))
    return mu_, sg_, mm_, vm_, ms_, vs_


def dropout_threshold(keep: float) -> int:
    return int(_load().update_oracle_dropout_threshold(float(keep)))


def dropout_forward(mu, words, keep: float) -> np.ndarray:
    """w[s,i] = mu[i] * (words[s,i] < threshold(keep)) / keep, fp64 [S_loc, N]; words uint32 [S_loc, >=N]."""
    mu = _f32(mu, "mu")
    words = np.ascontiguousarray(words, dtype=np.uint32)
    n, s = mu.shape[0], words.shape[0]
    w = np.empty((s, n), dtype=np.float64)
    _load().update_oracle_dropout_forward(n, words.shape[1], s, float(keep), _fptr(mu),
                                          words.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), _dptr(w))
    return w


def dropout_backward(G, words, keep: float, s_total: int, n: int = None, reduce_mean: bool = False) -> np.ndarray:
    """grad_mu[i] = g * sum_s G[s,i] * mask[s,i] / keep, fp64 [N]."""
    G = _f32(G, "G")
    words = np.ascontiguousarray(words, dtype=np.uint32)
    n = G.shape[1] if n is None else n
    out = np.empty(n, dtype=np.float64)
    _load().update_oracle_dropout_backward(n, G.shape[1], words.shape[1], G.shape[0], int(s_total),
                                           1 if reduce_mean else 0, float(keep), _fptr(G),
                                           words.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), _dptr(out))
    return out
