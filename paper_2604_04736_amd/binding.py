"""Python marshalling for the C ABI of libhot (declared in include/hot.h).

Same names as the C entry points.  This layer checks tensor metadata and passes raw
device pointers and the current HIP stream; every step of the path runs in the HIP
kernels.  There is no fallback: if libhot.so is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # imported before libhot.so so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhot.so")

HOT_OK, HOT_EINVAL, HOT_ENOMEM, HOT_EHIP, HOT_ERANGE = 0, -1, -2, -3, -4
HOT_STATIC_MAX_WEIGHTS = 1 << 28
HOT_REDUCE_SUM, HOT_REDUCE_MEAN, HOT_REDUCE_NONE = 0, 1, 2
HOT_KERNEL_FORWARD, HOT_KERNEL_BACKWARD, HOT_KERNEL_FORWARD_RNG, HOT_KERNEL_BACKWARD_RNG = 0, 1, 2, 3

EXPORTS = ("hot_create", "hot_forward", "hot_backward", "hot_destroy", "hot_set_launch",
           "hot_get_launch", "hot_last_hip_error", "hot_strerror", "hot_recommended_ld",
           "hot_version", "hot_probe_copy", "hot_forward_rng", "hot_backward_rng",
           "hot_sample_eps", "hot_sample_bits", "hot_probe_streams", "hot_stats_local",
           "hot_stats_merge", "hot_linear_forward_rng", "hot_adam_step", "hot_forward_dropout_rng",
           "hot_backward_dropout_rng", "hot_backward_rows", "hot_backward_adam",
           "hot_linear_backward_rng", "hot_kl", "hot_forward_dropout_units_rng",
           "hot_backward_dropout_units_rng", "hot_stats_whole", "hot_adam_forward", "hot_backward_adam_forward",
           "hot_linear_backward_rng_ws", "hot_linear_backward_workspace_bytes", "hot_forward_static",
           "hot_linear_launch_shape")


# Return types of the entry points that do not return an int status (as declared in include/hot.h).
RESTYPES = {"hot_strerror": ctypes.c_char_p, "hot_recommended_ld": ctypes.c_int64,
            "hot_linear_backward_workspace_bytes": ctypes.c_int64}


class hot_desc(ctypes.Structure):
    _fields_ = [("n_weights", ctypes.c_int64), ("ld", ctypes.c_int64),
                ("s_local", ctypes.c_int32), ("s_total", ctypes.c_int32),
                ("dataset_size", ctypes.c_double), ("device", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class hot_launch(ctypes.Structure):
    _fields_ = [("grid_blocks", ctypes.c_int32), ("chunks", ctypes.c_int32),
                ("unroll", ctypes.c_int32), ("nontemporal", ctypes.c_int32)]


class hot_rng(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("step", ctypes.c_uint32), ("first_sample", ctypes.c_uint32)]


class hot_linear_desc(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("in_features", ctypes.c_int64), ("out_features", ctypes.c_int64),
                ("ldx", ctypes.c_int64), ("weight_offset", ctypes.c_int64), ("bias_offset", ctypes.c_int64),
                ("s_local", ctypes.c_int32), ("reserved", ctypes.c_int32), ("x_sample_stride", ctypes.c_int64)]


class hot_adam(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("grad_scale", ctypes.c_double), ("sigma_min", ctypes.c_double),
                ("step", ctypes.c_int64)]


class HotError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code, self.hip = code, hip
        msg = lib().hot_strerror(code).decode()
        super().__init__(f"{where}: {msg} (code {code}" + (f", hipError {hip})" if hip else ")"))


_lib = None


def lib() -> ctypes.CDLL:
    """Opens libhot.so (built in-tree by paper_2604_04736_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run __graft_entry__.build() first")
    L = ctypes.CDLL(LIB_PATH)
    vp, fp = ctypes.c_void_p, ctypes.c_void_p
    L.hot_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(hot_desc)]
    L.hot_forward.argtypes = [vp, fp, fp, fp, fp, vp, vp]
    L.hot_backward.argtypes = [vp, fp, fp, fp, fp, fp, fp, vp]
    L.hot_kl.argtypes = [vp, fp, fp, vp, vp]
    L.hot_forward_static.argtypes = [ctypes.POINTER(hot_desc), fp, fp, fp, fp, vp, vp]
    L.hot_destroy.argtypes = [vp]
    rp = ctypes.POINTER(hot_rng)
    L.hot_forward_rng.argtypes = [vp, rp, fp, fp, fp, vp, vp]
    L.hot_backward_rng.argtypes = [vp, rp, fp, fp, fp, fp, fp, vp]
    L.hot_backward_rows.argtypes = [vp, rp, fp, fp, fp, fp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                    ctypes.c_int32, fp, fp, vp]
    L.hot_sample_eps.argtypes = [vp, rp, fp, vp]
    L.hot_sample_bits.argtypes = [vp, rp, vp, vp]
    L.hot_set_launch.argtypes = [vp, ctypes.c_int, ctypes.POINTER(hot_launch)]
    L.hot_get_launch.argtypes = [vp, ctypes.c_int, ctypes.POINTER(hot_launch)]
    L.hot_last_hip_error.argtypes = [vp]
    L.hot_strerror.argtypes = [ctypes.c_int]
    L.hot_strerror.restype = ctypes.c_char_p
    L.hot_recommended_ld.argtypes = [ctypes.c_int64]
    L.hot_recommended_ld.restype = ctypes.c_int64
    L.hot_version.argtypes = []
    L.hot_probe_copy.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int, vp]
    L.hot_probe_copy.restype = ctypes.c_int
    L.hot_probe_streams.argtypes = [vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, vp]
    L.hot_probe_streams.restype = ctypes.c_int
    L.hot_linear_forward_rng.argtypes = [ctypes.POINTER(hot_linear_desc), rp, fp, fp, fp, fp, fp, fp, vp]
    L.hot_linear_forward_rng.restype = ctypes.c_int
    L.hot_adam_step.argtypes = [ctypes.POINTER(hot_adam), ctypes.c_int64] + [fp] * 8 + [vp]
    L.hot_adam_step.restype = ctypes.c_int
    L.hot_linear_backward_rng.argtypes = [ctypes.POINTER(hot_linear_desc), ctypes.c_int32, ctypes.c_double, ctypes.c_uint32,
                                          rp] + [fp] * 11 + [vp]
    L.hot_linear_backward_rng_ws.argtypes = [ctypes.POINTER(hot_linear_desc), ctypes.c_int32, ctypes.c_double, ctypes.c_uint32,
                                             rp] + [fp] * 11 + [vp, ctypes.c_int64, vp]
    L.hot_linear_backward_rng_ws.restype = ctypes.c_int
    L.hot_linear_backward_workspace_bytes.argtypes = [ctypes.POINTER(hot_linear_desc)]
    L.hot_linear_launch_shape.argtypes = [ctypes.POINTER(hot_linear_desc), ctypes.c_int]
    L.hot_linear_backward_workspace_bytes.restype = ctypes.c_int64
    L.hot_adam_forward.argtypes = [vp, rp, ctypes.POINTER(hot_adam)] + [fp] * 10 + [vp, vp]
    L.hot_backward_adam.argtypes = [vp, rp, ctypes.POINTER(hot_adam)] + [fp] * 8 + [vp]
    L.hot_backward_adam_forward.argtypes = [vp, rp, rp, ctypes.POINTER(hot_adam)] + [fp] * 8 + [vp, vp]
    L.hot_forward_dropout_rng.argtypes = [ctypes.POINTER(hot_desc), rp, ctypes.c_double, fp, fp, vp]
    L.hot_forward_dropout_rng.restype = ctypes.c_int
    L.hot_backward_dropout_rng.argtypes = [ctypes.POINTER(hot_desc), rp, ctypes.c_double, fp, fp, vp]
    L.hot_backward_dropout_rng.restype = ctypes.c_int
    L.hot_forward_dropout_units_rng.argtypes = [ctypes.POINTER(hot_desc), rp, ctypes.c_double, ctypes.c_int64, ctypes.c_int64,
                                                fp, fp, vp]
    L.hot_backward_dropout_units_rng.argtypes = [ctypes.POINTER(hot_desc), rp, ctypes.c_double, ctypes.c_int64,
                                                 ctypes.c_int64, fp, fp, vp]
    L.hot_stats_local.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, vp, vp, vp]
    L.hot_stats_local.restype = ctypes.c_int
    L.hot_stats_whole.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, vp, vp, vp]
    L.hot_stats_merge.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, ctypes.c_int64,
                                  ctypes.c_int64, ctypes.c_int32, vp, vp, vp]
    L.hot_stats_merge.restype = ctypes.c_int
    for name in EXPORTS:
        if name not in RESTYPES:
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


class Plan:
    """Handle of a hot_plan plus the description it was made from."""

    def __init__(self, handle: int, desc: hot_desc):
        self.handle = ctypes.c_void_p(handle)
        self.desc = desc

    def __del__(self):
        try:
            hot_destroy(self)
        except Exception:
            pass


def _check(code: int, where: str, plan: Optional[Plan] = None):
    if code != HOT_OK:
        hip = lib().hot_last_hip_error(plan.handle) if plan is not None and plan.handle else 0
        raise HotError(code, where, hip)


def _check_planless(code: int, where: str):
    """For the entry points that take no plan: the HIP error is the calling thread's last one."""
    if code != HOT_OK:
        raise HotError(code, where, lib().hot_last_hip_error(None) if code == HOT_EHIP else 0)


def hot_version() -> int:
    return lib().hot_version()


def hot_strerror(code: int) -> str:
    return lib().hot_strerror(code).decode()


def hot_recommended_ld(n_weights: int) -> int:
    return int(lib().hot_recommended_ld(n_weights))


def hot_create(n_weights: int, ld: int, s_local: int, s_total: int, dataset_size: float,
               device: int = 0, flags: int = HOT_REDUCE_SUM) -> Plan:
    d = hot_desc(n_weights, ld, s_local, s_total, dataset_size, device, flags)
    out = ctypes.c_void_p()
    code = lib().hot_create(ctypes.byref(out), ctypes.byref(d))
    if code != HOT_OK:
        raise HotError(code, "hot_create")
    return Plan(out.value, d)


def hot_destroy(plan: Plan) -> None:
    if plan is not None and plan.handle:
        h, plan.handle = plan.handle, ctypes.c_void_p()
        code = lib().hot_destroy(h)
        if code != HOT_OK:
            raise HotError(code, "hot_destroy")


def hot_set_launch(plan: Plan, kernel: int, grid_blocks: int = 0, chunks: int = 0,
                   unroll: int = 0, nontemporal: int = 0) -> None:
    cfg = hot_launch(grid_blocks, chunks, unroll, nontemporal)
    _check(lib().hot_set_launch(plan.handle, kernel, ctypes.byref(cfg)), "hot_set_launch", plan)


def hot_get_launch(plan: Plan, kernel: int) -> dict:
    cfg = hot_launch()
    _check(lib().hot_get_launch(plan.handle, kernel, ctypes.byref(cfg)), "hot_get_launch", plan)
    return {k: getattr(cfg, k) for k, _ in hot_launch._fields_}


def _vec(t: torch.Tensor, n: int, dev: int, name: str) -> int:
    if not (t.is_cuda and t.device.index == dev and t.dtype == torch.float32):
        raise TypeError(f"{name}: need a float32 tensor on cuda:{dev}")
    if t.dim() != 1 or t.shape[0] != n or t.stride(0) != 1:
        raise ValueError(f"{name}: need a dense vector of {n} floats, got {tuple(t.shape)}")
    return t.data_ptr()


def _mat(t: torch.Tensor, s: int, n: int, ld: int, dev: int, name: str) -> int:
    if not (t.is_cuda and t.device.index == dev and t.dtype == torch.float32):
        raise TypeError(f"{name}: need a float32 tensor on cuda:{dev}")
    if t.dim() != 2 or t.shape[0] != s or not (n <= t.shape[1] <= ld) or t.stride(1) != 1 or \
            (s > 1 and t.stride(0) != ld):
        raise ValueError(f"{name}: need [S_loc={s}, >= {n}] rows with pitch {ld}, got "
                         f"{tuple(t.shape)} strides {t.stride()}")
    return t.data_ptr()


def _stream(dev: int) -> int:
    return torch.cuda.current_stream(dev).cuda_stream


def hot_forward(plan: Plan, mu, sigma, eps, w, kl_out=None) -> None:
    """w[s,i] = mu[i] + sigma[i]*eps[s,i]; kl_out (one float64 on the device) gets the KL term."""
    d = plan.desc
    klp = _kl_ptr(plan, kl_out)
    code = lib().hot_forward(plan.handle,
                             _vec(mu, d.n_weights, d.device, "mu"),
                             _vec(sigma, d.n_weights, d.device, "sigma"),
                             _mat(eps, d.s_local, d.n_weights, d.ld, d.device, "eps"),
                             _mat(w, d.s_local, d.n_weights, d.ld, d.device, "w"),
                             klp, _stream(d.device))
    _check(code, "hot_forward", plan)


def hot_forward_static(desc: hot_desc, mu, sigma, eps, w, kl_out=None) -> None:
    """hot_forward without a plan and without any allocation (see include/hot.h); desc: a hot_desc."""
    d = desc
    klp = None
    if kl_out is not None:
        if not (kl_out.is_cuda and kl_out.device.index == d.device and kl_out.dtype == torch.float64 and kl_out.numel() == 1):
            raise TypeError("kl_out: need one float64 element on desc.device")
        klp = kl_out.data_ptr()
    code = lib().hot_forward_static(ctypes.byref(d),
                                    _vec(mu, d.n_weights, d.device, "mu"),
                                    _vec(sigma, d.n_weights, d.device, "sigma"),
                                    _mat(eps, d.s_local, d.n_weights, d.ld, d.device, "eps"),
                                    _mat(w, d.s_local, d.n_weights, d.ld, d.device, "w"),
                                    klp, _stream(d.device))
    _check_planless(code, "hot_forward_static")


def hot_backward(plan: Plan, mu, sigma, eps, grad_w, grad_mu, grad_sigma) -> None:
    """grad_mu, grad_sigma from the per-sample weight gradients grad_w (see include/hot.h)."""
    d = plan.desc
    code = lib().hot_backward(plan.handle,
                              _vec(mu, d.n_weights, d.device, "mu"),
                              _vec(sigma, d.n_weights, d.device, "sigma"),
                              _mat(eps, d.s_local, d.n_weights, d.ld, d.device, "eps"),
                              _mat(grad_w, d.s_local, d.n_weights, d.ld, d.device, "grad_w"),
                              _vec(grad_mu, d.n_weights, d.device, "grad_mu"),
                              _vec(grad_sigma, d.n_weights, d.device, "grad_sigma"),
                              _stream(d.device))
    _check(code, "hot_backward", plan)


def _kl_ptr(plan: Plan, kl_out):
    if kl_out is None:
        return None
    d = plan.desc
    if not (kl_out.is_cuda and kl_out.device.index == d.device and kl_out.dtype == torch.float64
            and kl_out.numel() == 1):
        raise TypeError("kl_out: need one float64 element on the plan's device")
    return kl_out.data_ptr()


def hot_forward_rng(plan: Plan, rng: hot_rng, mu, sigma, w, kl_out=None) -> None:
    """hot_forward with eps drawn in the kernel (see hot_rng in include/hot.h)."""
    d = plan.desc
    code = lib().hot_forward_rng(plan.handle, ctypes.byref(rng),
                                 _vec(mu, d.n_weights, d.device, "mu"),
                                 _vec(sigma, d.n_weights, d.device, "sigma"),
                                 _mat(w, d.s_local, d.n_weights, d.ld, d.device, "w"),
                                 _kl_ptr(plan, kl_out), _stream(d.device))
    _check(code, "hot_forward_rng", plan)


def hot_backward_rng(plan: Plan, rng: hot_rng, mu, sigma, grad_w, grad_mu, grad_sigma) -> None:
    """hot_backward with eps regenerated in the kernel."""
    d = plan.desc
    code = lib().hot_backward_rng(plan.handle, ctypes.byref(rng),
                                  _vec(mu, d.n_weights, d.device, "mu"),
                                  _vec(sigma, d.n_weights, d.device, "sigma"),
                                  _mat(grad_w, d.s_local, d.n_weights, d.ld, d.device, "grad_w"),
                                  _vec(grad_mu, d.n_weights, d.device, "grad_mu"),
                                  _vec(grad_sigma, d.n_weights, d.device, "grad_sigma"),
                                  _stream(d.device))
    _check(code, "hot_backward_rng", plan)


def hot_sample_eps(plan: Plan, rng: hot_rng, eps) -> None:
    """Writes the fp32 draw eps[S_loc, ld] the *_rng calls use."""
    d = plan.desc
    code = lib().hot_sample_eps(plan.handle, ctypes.byref(rng),
                                _mat(eps, d.s_local, d.n_weights, d.ld, d.device, "eps"), _stream(d.device))
    _check(code, "hot_sample_eps", plan)


def hot_sample_bits(plan: Plan, rng: hot_rng, bits) -> None:
    """Writes the raw generator words as int32 bit patterns, [S_loc, ld]."""
    d = plan.desc
    if not (bits.is_cuda and bits.device.index == d.device and bits.dtype == torch.int32 and bits.dim() == 2
            and bits.shape[0] == d.s_local and d.n_weights <= bits.shape[1] <= d.ld and bits.stride(1) == 1
            and (d.s_local == 1 or bits.stride(0) == d.ld)):
        raise ValueError("bits: need an int32 [S_loc, >= N] tensor with pitch ld on the plan's device")
    code = lib().hot_sample_bits(plan.handle, ctypes.byref(rng), bits.data_ptr(), _stream(d.device))
    _check(code, "hot_sample_bits", plan)


def hot_probe_copy(dst: torch.Tensor, src: torch.Tensor, nontemporal: int = 0) -> None:
    """Plain device copy of src into dst (measurement aid, see include/hot.h)."""
    if not (dst.is_cuda and src.is_cuda and dst.device == src.device and dst.is_contiguous()
            and src.is_contiguous() and dst.numel() * dst.element_size() == src.numel() * src.element_size()):
        raise ValueError("hot_probe_copy: need two contiguous device tensors of equal byte size")
    with torch.cuda.device(src.device):
        code = lib().hot_probe_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(),
                                    nontemporal, _stream(src.device.index))
    _check_planless(code, "hot_probe_copy")


def hot_probe_streams(arena: torch.Tensor, stream_bytes: int, reads: int, writes: int) -> None:
    """reads read streams + writes write streams of stream_bytes each inside arena (see include/hot.h)."""
    if not (arena.is_cuda and arena.is_contiguous()
            and arena.numel() * arena.element_size() >= (reads + writes) * stream_bytes):
        raise ValueError("hot_probe_streams: arena too small or not a contiguous device tensor")
    with torch.cuda.device(arena.device):
        code = lib().hot_probe_streams(arena.data_ptr(), stream_bytes, reads, writes, _stream(arena.device.index))
    _check_planless(code, "hot_probe_streams")


def _dense2(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.dtype == dtype and t.dim() == 2 and t.stride(1) == 1):
        raise TypeError(f"{name}: need a 2-D {dtype} device tensor with unit column stride")
    return t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else t.shape[1])


def hot_stats_local(yhat: torch.Tensor, mean: torch.Tensor, m2: torch.Tensor) -> None:
    """(mean, M2) over the rows of yhat[S_loc, M] into fp64 vectors mean[M], m2[M]."""
    s_loc, m, ld = _dense2(yhat, torch.float32, "yhat")
    for t, name in ((mean, "mean"), (m2, "m2")):
        if not (t.is_cuda and t.device == yhat.device and t.dtype == torch.float64 and t.dim() == 1
                and t.shape[0] == m and t.stride(0) == 1):
            raise TypeError(f"{name}: need a dense float64 vector of {m} elements on {yhat.device}")
    with torch.cuda.device(yhat.device):
        code = lib().hot_stats_local(yhat.data_ptr(), m, ld, s_loc, mean.data_ptr(), m2.data_ptr(),
                                     _stream(yhat.device.index))
    _check_planless(code, "hot_stats_local")


def hot_stats_merge(means: torch.Tensor, m2s: torch.Tensor, counts, ddof: int, mean_out: torch.Tensor,
                    std_out: torch.Tensor) -> None:
    """Pooled mean / std from the partials means[parts, M], m2s[parts, M] with counts[parts]."""
    parts, m, ld = _dense2(means, torch.float64, "means")
    if _dense2(m2s, torch.float64, "m2s") != (parts, m, ld) or m2s.device != means.device:
        raise ValueError("m2s must match means in shape, pitch and device")
    if len(counts) != parts:
        raise ValueError("counts must have one entry per partial")
    for t, name in ((mean_out, "mean_out"), (std_out, "std_out")):
        if not (t.is_cuda and t.device == means.device and t.dtype == torch.float32 and t.dim() == 1
                and t.shape[0] == m and t.stride(0) == 1):
            raise TypeError(f"{name}: need a dense float32 vector of {m} elements on {means.device}")
    c = (ctypes.c_int32 * parts)(*[int(v) for v in counts])
    with torch.cuda.device(means.device):
        code = lib().hot_stats_merge(means.data_ptr(), m2s.data_ptr(), c, parts, m, ld, int(ddof),
                                     mean_out.data_ptr(), std_out.data_ptr(), _stream(means.device.index))
    _check_planless(code, "hot_stats_merge")


def hot_linear_forward_rng(rng: hot_rng, x, mu_w, sigma_w, mu_b, sigma_b, y, weight_offset: int = 0,
                           bias_offset: int = 0) -> None:
    """y[S, R, O] = x_s (mu_w + sigma_w*eps_s)^T + (mu_b + sigma_b*eps_s^b), eps drawn in the kernel;
    x is [R, K] (shared by the samples) or [S, R, K] (one input per sample)."""
    def chk(t, shape, name):
        if not (t.is_cuda and t.device == x.device and t.dtype == torch.float32 and tuple(t.shape) == shape
                and t.is_contiguous()):
            raise TypeError(f"{name}: need a contiguous float32 tensor of shape {shape} on {x.device}")
    if not (x.is_cuda and x.dtype == torch.float32 and x.dim() in (2, 3) and x.stride(-1) == 1):
        raise TypeError("x: need a [rows, K] or [S_loc, rows, K] float32 device tensor with unit column stride")
    rows, k = x.shape[-2:]
    ldx = x.stride(-2) if rows > 1 else k
    x_stride = 0
    if x.dim() == 3:
        if y.dim() != 3 or x.shape[0] != y.shape[0]:
            raise ValueError("per-sample x needs as many [rows, K] blocks as y has samples")
        x_stride = x.stride(0) if x.shape[0] > 1 else rows * ldx
    if mu_w.dim() != 2 or mu_w.shape[1] != k:
        raise ValueError("mu_w must be [out_features, in_features]")
    o = mu_w.shape[0]
    chk(mu_w, (o, k), "mu_w")
    chk(sigma_w, (o, k), "sigma_w")
    if (mu_b is None) != (sigma_b is None):
        raise ValueError("give both bias arrays or neither")
    if mu_b is not None:
        chk(mu_b, (o,), "mu_b")
        chk(sigma_b, (o,), "sigma_b")
    if y.dim() != 3:
        raise ValueError("y must be [S_loc, rows, out_features]")
    s_loc = y.shape[0]
    chk(y, (s_loc, rows, o), "y")
    d = hot_linear_desc(rows, k, o, ldx, weight_offset, bias_offset, s_loc, 0, x_stride)
    with torch.cuda.device(x.device):
        code = lib().hot_linear_forward_rng(ctypes.byref(d), ctypes.byref(rng), x.data_ptr(), mu_w.data_ptr(),
                                            sigma_w.data_ptr(), mu_b.data_ptr() if mu_b is not None else None,
                                            sigma_b.data_ptr() if mu_b is not None else None, y.data_ptr(),
                                            _stream(x.device.index))
    _check_planless(code, "hot_linear_forward_rng")


def hot_adam_step(params: hot_adam, mu, sigma, grad_mu, grad_sigma, m_mu, v_mu, m_sigma, v_sigma) -> None:
    """One in-place Adam step on (mu, sigma) and their moment arrays (see include/hot.h)."""
    n = mu.shape[0]
    dev = mu.device.index
    ptrs = [_vec(t, n, dev, name) for t, name in ((mu, "mu"), (sigma, "sigma"), (grad_mu, "grad_mu"),
                                                   (grad_sigma, "grad_sigma"), (m_mu, "m_mu"), (v_mu, "v_mu"),
                                                   (m_sigma, "m_sigma"), (v_sigma, "v_sigma"))]
    with torch.cuda.device(mu.device):
        code = lib().hot_adam_step(ctypes.byref(params), n, *ptrs, _stream(dev))
    _check_planless(code, "hot_adam_step")


def hot_forward_dropout_rng(plan: Plan, rng: hot_rng, keep: float, mu, w) -> None:
    """w[s,i] = mu[i] * mask[s,i] / keep with the mask drawn in the kernel."""
    d = plan.desc
    with torch.cuda.device(d.device):
        code = lib().hot_forward_dropout_rng(ctypes.byref(d), ctypes.byref(rng), float(keep),
                                             _vec(mu, d.n_weights, d.device, "mu"),
                                             _mat(w, d.s_local, d.n_weights, d.ld, d.device, "w"), _stream(d.device))
    _check_planless(code, "hot_forward_dropout_rng")


def hot_backward_dropout_rng(plan: Plan, rng: hot_rng, keep: float, grad_w, grad_mu) -> None:
    """grad_mu[i] = g * sum_s grad_w[s,i] * mask[s,i] / keep with the mask regenerated in the kernel."""
    d = plan.desc
    with torch.cuda.device(d.device):
        code = lib().hot_backward_dropout_rng(ctypes.byref(d), ctypes.byref(rng), float(keep),
                                              _mat(grad_w, d.s_local, d.n_weights, d.ld, d.device, "grad_w"),
                                              _vec(grad_mu, d.n_weights, d.device, "grad_mu"), _stream(d.device))
    _check_planless(code, "hot_backward_dropout_rng")


def hot_backward_rows(plan: Plan, rng, mu, sigma, eps, grad_w, first_row: int, accumulate: bool, add_kl: bool,
                      grad_mu, grad_sigma) -> None:
    """hot_backward over the local samples first_row .. first_row + grad_w.shape[0] - 1 only (see hot.h)."""
    d = plan.desc
    rows = grad_w.shape[0]
    if (rng is None) == (eps is None):
        raise ValueError("give exactly one of rng and eps")
    code = lib().hot_backward_rows(plan.handle, ctypes.byref(rng) if rng is not None else None,
                                   _vec(mu, d.n_weights, d.device, "mu"), _vec(sigma, d.n_weights, d.device, "sigma"),
                                   _mat(eps, rows, d.n_weights, d.ld, d.device, "eps") if eps is not None else None,
                                   _mat(grad_w, rows, d.n_weights, d.ld, d.device, "grad_w"), first_row, rows,
                                   1 if accumulate else 0, 1 if add_kl else 0,
                                   _vec(grad_mu, d.n_weights, d.device, "grad_mu"),
                                   _vec(grad_sigma, d.n_weights, d.device, "grad_sigma"), _stream(d.device))
    _check(code, "hot_backward_rows", plan)


def hot_backward_adam(plan: Plan, rng, params: hot_adam, mu, sigma, eps, grad_w, m_mu, v_mu, m_sigma, v_sigma) -> None:
    """hot_backward and hot_adam_step in one pass for a plan that holds all S samples (see include/hot.h)."""
    d = plan.desc
    if (rng is None) == (eps is None):
        raise ValueError("give exactly one of rng and eps")
    n, dev = d.n_weights, d.device
    code = lib().hot_backward_adam(plan.handle, ctypes.byref(rng) if rng is not None else None, ctypes.byref(params),
                                   _vec(mu, n, dev, "mu"), _vec(sigma, n, dev, "sigma"),
                                   _mat(eps, d.s_local, n, d.ld, dev, "eps") if eps is not None else None,
                                   _mat(grad_w, d.s_local, n, d.ld, dev, "grad_w"),
                                   _vec(m_mu, n, dev, "m_mu"), _vec(v_mu, n, dev, "v_mu"),
                                   _vec(m_sigma, n, dev, "m_sigma"), _vec(v_sigma, n, dev, "v_sigma"), _stream(dev))
    _check(code, "hot_backward_adam", plan)


def hot_linear_backward_workspace_bytes(rows: int, in_features: int, out_features: int, s_local: int) -> int:
    """Bytes of device scratch with which hot_linear_backward_rng(..., workspace=...) splits the rows of this
    layer shape over workgroups as far as it wants to; 0 if it would not use any."""
    d = hot_linear_desc(rows, in_features, out_features, in_features, 0, 0, s_local, 0, 0)
    n = lib().hot_linear_backward_workspace_bytes(ctypes.byref(d))
    if n < 0:
        _check_planless(int(n), "hot_linear_backward_workspace_bytes")
    return int(n)


def hot_linear_launch_shape(rows: int, in_features: int, out_features: int, s_local: int, which: int, per_sample_x: bool = False,
                            ldx: int = 0) -> int:
    """Code of the launch shape hot_linear_forward_rng (which = 0) or the input-gradient part of
    hot_linear_backward_rng (which = 1) chooses for this layer; which = 2: of the kernel that takes both gradients in
    one pass (hot_linear_backward_rng_ws with dx and a full workspace); see include/hot.h.  0: the other kernels."""
    ldx = ldx or in_features
    d = hot_linear_desc(rows, in_features, out_features, ldx, 0, 0, s_local, 0, rows * ldx if per_sample_x else 0)
    code = lib().hot_linear_launch_shape(ctypes.byref(d), which)
    if code < 0:
        _check_planless(int(code), "hot_linear_launch_shape")
    return int(code)


def hot_linear_backward_rng(rng: hot_rng, x, dy, mu_w, sigma_w, mu_b, sigma_b, grad_mu_w, grad_sigma_w, grad_mu_b,
                            grad_sigma_b, dx, s_total: int, dataset_size: float, flags: int = HOT_REDUCE_SUM,
                            weight_offset: int = 0, bias_offset: int = 0, workspace=None) -> None:
    """Gradients of the sampled linear layer from dy [S_loc, R, O] (see include/hot.h): weight and bias
    gradients scaled like hot_backward's, and dx [S_loc, R, K] (or None to skip it).  workspace: an optional
    contiguous device tensor (any dtype) used as scratch (hot_linear_backward_rng_ws)."""
    def chk(t, shape, name):
        if not (t.is_cuda and t.device == x.device and t.dtype == torch.float32 and tuple(t.shape) == shape
                and t.is_contiguous()):
            raise TypeError(f"{name}: need a contiguous float32 tensor of shape {shape} on {x.device}")
    if not (x.is_cuda and x.dtype == torch.float32 and x.dim() in (2, 3) and x.stride(-1) == 1):
        raise TypeError("x: need a [rows, K] or [S_loc, rows, K] float32 device tensor with unit column stride")
    rows, k = x.shape[-2:]
    ldx = x.stride(-2) if rows > 1 else k
    if dy.dim() != 3:
        raise ValueError("dy must be [S_loc, rows, out_features]")
    s_loc, o = dy.shape[0], dy.shape[2]
    x_stride = 0
    if x.dim() == 3:
        if x.shape[0] != s_loc:
            raise ValueError("per-sample x needs as many [rows, K] blocks as dy has samples")
        x_stride = x.stride(0) if s_loc > 1 else rows * ldx
    chk(dy, (s_loc, rows, o), "dy")
    for t, name in ((mu_w, "mu_w"), (sigma_w, "sigma_w"), (grad_mu_w, "grad_mu_w"), (grad_sigma_w, "grad_sigma_w")):
        chk(t, (o, k), name)
    bias = (mu_b, sigma_b, grad_mu_b, grad_sigma_b)
    if any(b is None for b in bias) and not all(b is None for b in bias):
        raise ValueError("give all four bias arrays or none")
    if mu_b is not None:
        for t, name in zip(bias, ("mu_b", "sigma_b", "grad_mu_b", "grad_sigma_b")):
            chk(t, (o,), name)
    if dx is not None:
        chk(dx, (s_loc, rows, k), "dx")
    d = hot_linear_desc(rows, k, o, ldx, weight_offset, bias_offset, s_loc, 0, x_stride)
    ptr = lambda t: t.data_ptr() if t is not None else None
    if workspace is not None and not (workspace.is_cuda and workspace.device == x.device and workspace.is_contiguous()):
        raise TypeError(f"workspace: need a contiguous tensor on {x.device}")
    with torch.cuda.device(x.device):
        if workspace is None:
            code = lib().hot_linear_backward_rng(ctypes.byref(d), int(s_total), float(dataset_size), int(flags), ctypes.byref(rng),
                                                 x.data_ptr(), dy.data_ptr(), mu_w.data_ptr(), sigma_w.data_ptr(), ptr(mu_b),
                                                 ptr(sigma_b), grad_mu_w.data_ptr(), grad_sigma_w.data_ptr(), ptr(grad_mu_b),
                                                 ptr(grad_sigma_b), ptr(dx), _stream(x.device.index))
        else:
            code = lib().hot_linear_backward_rng_ws(ctypes.byref(d), int(s_total), float(dataset_size), int(flags), ctypes.byref(rng),
                                                    x.data_ptr(), dy.data_ptr(), mu_w.data_ptr(), sigma_w.data_ptr(), ptr(mu_b),
                                                    ptr(sigma_b), grad_mu_w.data_ptr(), grad_sigma_w.data_ptr(), ptr(grad_mu_b),
                                                    ptr(grad_sigma_b), ptr(dx), workspace.data_ptr(),
                                                    workspace.numel() * workspace.element_size(), _stream(x.device.index))
    _check_planless(code, "hot_linear_backward_rng_ws" if workspace is not None else "hot_linear_backward_rng")


def hot_kl(plan: Plan, mu, sigma, kl_out) -> None:
    """kl_out (one float64 on the device) = the KL term of (mu, sigma), without forming w."""
    d = plan.desc
    code = lib().hot_kl(plan.handle, _vec(mu, d.n_weights, d.device, "mu"), _vec(sigma, d.n_weights, d.device, "sigma"),
                        _kl_ptr(plan, kl_out), _stream(d.device))
    _check(code, "hot_kl", plan)


def hot_forward_dropout_units_rng(plan: Plan, rng: hot_rng, keep: float, in_features: int, unit_offset: int, mu, w) -> None:
    """w[s,i] = mu[i] * mask[s, i mod in_features] / keep: one Bernoulli variable per input unit and sample."""
    d = plan.desc
    with torch.cuda.device(d.device):
        code = lib().hot_forward_dropout_units_rng(ctypes.byref(d), ctypes.byref(rng), float(keep), int(in_features),
                                                   int(unit_offset), _vec(mu, d.n_weights, d.device, "mu"),
                                                   _mat(w, d.s_local, d.n_weights, d.ld, d.device, "w"), _stream(d.device))
    _check_planless(code, "hot_forward_dropout_units_rng")


def hot_backward_dropout_units_rng(plan: Plan, rng: hot_rng, keep: float, in_features: int, unit_offset: int, grad_w,
                                   grad_mu) -> None:
    """grad_mu[i] = g * sum_s grad_w[s,i] * mask[s, i mod in_features] / keep."""
    d = plan.desc
    with torch.cuda.device(d.device):
        code = lib().hot_backward_dropout_units_rng(ctypes.byref(d), ctypes.byref(rng), float(keep), int(in_features),
                                                    int(unit_offset),
                                                    _mat(grad_w, d.s_local, d.n_weights, d.ld, d.device, "grad_w"),
                                                    _vec(grad_mu, d.n_weights, d.device, "grad_mu"), _stream(d.device))
    _check_planless(code, "hot_backward_dropout_units_rng")


def hot_stats_whole(yhat: torch.Tensor, ddof: int, mean_out: torch.Tensor, std_out: torch.Tensor) -> None:
    """Mean and standard deviation over the rows of yhat[S, M] in one pass (all samples on this GPU)."""
    s, m, ld = _dense2(yhat, torch.float32, "yhat")
    for t, name in ((mean_out, "mean_out"), (std_out, "std_out")):
        if not (t.is_cuda and t.device == yhat.device and t.dtype == torch.float32 and t.dim() == 1
                and t.shape[0] == m and t.stride(0) == 1):
            raise TypeError(f"{name}: need a dense float32 vector of {m} elements on {yhat.device}")
    with torch.cuda.device(yhat.device):
        code = lib().hot_stats_whole(yhat.data_ptr(), m, ld, s, int(ddof), mean_out.data_ptr(), std_out.data_ptr(),
                                     _stream(yhat.device.index))
    _check_planless(code, "hot_stats_whole")


def hot_adam_forward(plan: Plan, rng, params: hot_adam, mu, sigma, grad_mu, grad_sigma, m_mu, v_mu, m_sigma, v_sigma,
                     eps, w, kl_out=None) -> None:
    """hot_adam_step and the next step's hot_forward / hot_forward_rng in one pass (see include/hot.h)."""
    d = plan.desc
    if (rng is None) == (eps is None):
        raise ValueError("give exactly one of rng and eps")
    n, dev = d.n_weights, d.device
    vecs = [_vec(t, n, dev, name) for t, name in ((mu, "mu"), (sigma, "sigma"), (grad_mu, "grad_mu"), (grad_sigma, "grad_sigma"),
                                                  (m_mu, "m_mu"), (v_mu, "v_mu"), (m_sigma, "m_sigma"), (v_sigma, "v_sigma"))]
    code = lib().hot_adam_forward(plan.handle, ctypes.byref(rng) if rng is not None else None, ctypes.byref(params), *vecs,
                                  _mat(eps, d.s_local, n, d.ld, dev, "eps") if eps is not None else None,
                                  _mat(w, d.s_local, n, d.ld, dev, "w"), _kl_ptr(plan, kl_out), _stream(dev))
    _check(code, "hot_adam_forward", plan)


def hot_backward_adam_forward(plan: Plan, rng: hot_rng, rng_next: hot_rng, params: hot_adam, mu, sigma, grad_w, m_mu, v_mu,
                              m_sigma, v_sigma, w, kl_out=None) -> None:
    """hot_backward_rng, hot_adam_step and the next step's hot_forward_rng in one pass (see include/hot.h)."""
    d = plan.desc
    n, dev = d.n_weights, d.device
    code = lib().hot_backward_adam_forward(plan.handle, ctypes.byref(rng), ctypes.byref(rng_next), ctypes.byref(params),
                                           _vec(mu, n, dev, "mu"), _vec(sigma, n, dev, "sigma"),
                                           _mat(grad_w, d.s_local, n, d.ld, dev, "grad_w"),
                                           _vec(m_mu, n, dev, "m_mu"), _vec(v_mu, n, dev, "v_mu"),
                                           _vec(m_sigma, n, dev, "m_sigma"), _vec(v_sigma, n, dev, "v_sigma"),
                                           _mat(w, d.s_local, n, d.ld, dev, "w"), _kl_ptr(plan, kl_out), _stream(dev))
    _check(code, "hot_backward_adam_forward", plan)
