"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the HIP library's callers and the CPU oracle's tests.  It
holds none of the method's arithmetic: it only fills mu, sigma, eps and G with
numbers.  Every element is a pure function of (seed, stream, element index) through
a counter-based hash, so any slice can be regenerated on its own, on the CPU or on
the GPU (torch integer ops are bit-identical on both; the floating-point stage may
differ in the last bit between devices, so a test always hands the very same bytes
to both sides).

Shapes (arxiv 2604.04736, section "Experimental Setup" and "Results"):
  C1  the use-case-2 MLP 96 -> 128 -> 128 -> 24 with biases, S = 16 over 4 GPUs;
  C2  the use-case-1 ViT (4x4 patches, width 192, 6 layers, MLP 768), S = 16 over 4 GPUs;
  C3  all 16 samples on one GPU (the fixed-sample baseline), 6 * 2^20 weights;
  C4  the use-case-3 SWIN model (> 200 million weights), two samples per GPU, S = 16;
  C5  adversarial: odd N, packed unaligned rows, S_loc = 13 of S = 52, values spread
      over many decades.
Value distributions: means Kaiming-normal per layer, std = sqrt(2 / fan_in); standard
deviations a constant inversely proportional to the layer width (sigma^2 = kappa /
fan_in, kappa = 0.01) with a small log-normal jitter so that all elements differ;
eps ~ N(0, 1); G ~ N(0, 1) (the paper fixes no distribution for the data-loss
gradients).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Tuple

import torch

STREAM_MU, STREAM_SIGMA, STREAM_EPS, STREAM_G, STREAM_AUX = 0, 1, 2, 3, 4

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

KAPPA = 0.01
SIGMA_JITTER = 0.25
CIFAR10_TRAIN_SIZE = 45_000.0   # 50k training images minus the 10 % held out for validation


def _signed(c: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant (torch has no uint64 maths)."""
    c &= _MASK64
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _signed(_M1)
    z = (z ^ _lsr(z, 27)) * _signed(_M2)
    return z ^ _lsr(z, 31)


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """64-bit key of one (seed, stream) pair."""
    return _mix_int(_mix_int(seed * _GOLDEN + 0x5851F42D4C957F2D) + stream * _GOLDEN + 1)


def hash64(seed: int, stream: int, counters: torch.Tensor) -> torch.Tensor:
    """SplitMix64 output number ``counter`` of the generator whose state starts at the key."""
    key = stream_key(seed, stream)
    state = (counters + 1) * _signed(_GOLDEN) + _signed(key)
    return _mix(state)


def _uniform(seed: int, stream: int, counters: torch.Tensor) -> torch.Tensor:
    """Uniform in the open interval (0, 1), fp64, from the top 52 bits."""
    h = hash64(seed, stream, counters)
    return (_lsr(h, 12).to(torch.float64) + 0.5) * (2.0 ** -52)


def uniform(seed: int, stream: int, start: int, count: int, device, lane: int = 0,
            lanes: int = 4) -> torch.Tensor:
    """Element k uses counter lanes*k + lane, so one element can own several draws."""
    k = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _uniform(seed, stream, k * lanes + lane)


def normal(seed: int, stream: int, start: int, count: int, device) -> torch.Tensor:
    """Standard normal by Box-Muller (lanes 0 and 1 of the element), fp64."""
    u1 = uniform(seed, stream, start, count, device, lane=0)
    u2 = uniform(seed, stream, start, count, device, lane=1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


# --------------------------------------------------------------------------- shapes

def _mlp_segments() -> List[Tuple[int, int]]:
    dims = [96, 128, 128, 24]
    seg = []
    for a, b in zip(dims[:-1], dims[1:]):
        seg += [(a * b, a), (b, a)]          # weight matrix, then bias
    return seg


def _vit_segments() -> List[Tuple[int, int]]:
    d, mlp, layers, patch_in, tokens, classes = 192, 768, 6, 4 * 4 * 3, 64 + 1, 10
    seg = [(patch_in * d, patch_in), (d, patch_in), (d, d), (tokens * d, d)]
    for _ in range(layers):
        seg += [(2 * d, d),
                (d * 3 * d, d), (3 * d, d),
                (d * d, d), (d, d),
                (2 * d, d),
                (d * mlp, d), (mlp, d),
                (mlp * d, mlp), (d, mlp)]
    seg += [(2 * d, d), (d * classes, d), (classes, d)]
    return seg


def _cycled_segments(n: int, pattern: List[Tuple[int, int]]) -> List[Tuple[int, int]]:
    seg, total, j = [], 0, 0
    while total < n:
        length, fan_in = pattern[j % len(pattern)]
        length = min(length, n - total)
        seg.append((length, fan_in))
        total += length
        j += 1
    return seg


def _c3_segments(n: int) -> List[Tuple[int, int]]:
    pattern = [(1 << 16, 192), (1 << 18, 384), (1 << 17, 192), (1 << 20, 768),
               (1 << 19, 576), (1 << 16, 768)]
    return _cycled_segments(n, pattern)


def _swin_segments(n: int) -> List[Tuple[int, int]]:
    e = 540
    pattern = [(e * 3 * e, e), (3 * e, e), (e * e, e), (e, e),
               (e * 4 * e, e), (4 * e, e), (4 * e * e, 4 * e), (e, 4 * e),
               (2 * e * 6 * e, 2 * e), (6 * e, 2 * e), (2 * e * 2 * e, 2 * e), (2 * e, 2 * e),
               (2 * e * 8 * e, 2 * e), (8 * e, 2 * e), (8 * e * 2 * e, 8 * e), (2 * e, 8 * e)]
    return _cycled_segments(n, pattern)


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    n_weights: int
    s_local: int
    s_total: int
    ld: int
    dataset_size: float
    kind: str                              # "paper" or "adversarial"
    segments: Tuple[Tuple[int, int], ...]  # (length, fan_in) per layer segment
    note: str

    @property
    def items(self) -> int:
        return self.n_weights * self.s_local


def _round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


def _make(name, seed, segs, s_local, s_total, padded, kind, note) -> Workload:
    n = sum(l for l, _ in segs)
    ld = _round_up(n, 64) if padded else n
    return Workload(name, seed, n, s_local, s_total, ld, CIFAR10_TRAIN_SIZE, kind,
                    tuple(segs), note)


def _configs() -> Dict[str, Workload]:
    c = {}
    c["C1"] = _make("C1", 0, _mlp_segments(), 4, 16, True, "paper",
                    "MLP 96-128-128-24, S=16 over 4 GPUs")
    c["C2"] = _make("C2", 1, _vit_segments(), 4, 16, True, "paper",
                    "ViT width 192 depth 6, S=16 over 4 GPUs")
    c["C3"] = _make("C3", 2, _c3_segments(6 << 20), 16, 16, False, "paper",
                    "6*2^20 weights, all 16 samples on one GPU")
    c["C4"] = _make("C4", 3, _swin_segments(200 << 20), 2, 16, False, "paper",
                    "SWIN-sized 200*2^20 weights, 2 samples per GPU of S=16")
    c["C5"] = _make("C5", 4, [(7_700_003, 1)], 13, 52, False, "adversarial",
                    "odd N, packed unaligned rows, S_loc=13 of S=52, many-decade values")
    return c


CONFIGS: Dict[str, Workload] = _configs()


def scaled(wl: Workload, n_weights: int, name: str = None) -> Workload:
    """The same recipe on the first ``n_weights`` weights (for oracle-sized test cases)."""
    segs = _cycled_segments(n_weights, list(wl.segments))
    n = sum(l for l, _ in segs)
    ld = n if wl.ld == wl.n_weights else _round_up(n, 64)
    return Workload(name or f"{wl.name}[:{n}]", wl.seed, n, wl.s_local, wl.s_total, ld,
                    wl.dataset_size, wl.kind, tuple(segs), wl.note)


# --------------------------------------------------------------------------- values

_CHUNK = 1 << 24


def _fan_in(wl: Workload, device) -> torch.Tensor:
    lengths = torch.tensor([l for l, _ in wl.segments], dtype=torch.int64, device=device)
    fans = torch.tensor([f for _, f in wl.segments], dtype=torch.float64, device=device)
    return torch.repeat_interleave(fans, lengths)


def _fill_rows(out: torch.Tensor, n: int, fn) -> None:
    """out[s, c0:c0+cnt] = fn(s, c0, cnt), chunked; logical element index is k = s*n + i."""
    for s in range(out.shape[0]):
        for c0 in range(0, n, _CHUNK):
            cnt = min(_CHUNK, n - c0)
            out[s, c0:c0 + cnt] = fn(s, c0, cnt).to(torch.float32)


def _paper_values(wl: Workload, device, mu, sigma, eps, G) -> None:
    n = wl.n_weights
    fan = _fan_in(wl, device)
    for c0 in range(0, n, _CHUNK):
        cnt = min(_CHUNK, n - c0)
        f = fan[c0:c0 + cnt]
        z = normal(wl.seed, STREAM_MU, c0, cnt, device)
        mu[c0:c0 + cnt] = (torch.sqrt(2.0 / f) * z).to(torch.float32)
        z = normal(wl.seed, STREAM_SIGMA, c0, cnt, device)
        sigma[c0:c0 + cnt] = (torch.sqrt(KAPPA / f) * torch.exp(SIGMA_JITTER * z)).to(torch.float32)
    _fill_rows(eps, n, lambda s, c0, cnt: normal(wl.seed, STREAM_EPS, s * n + c0, cnt, device))
    _fill_rows(G, n, lambda s, c0, cnt: normal(wl.seed, STREAM_G, s * n + c0, cnt, device))


def _adversarial_values(wl: Workload, device, mu, sigma, eps, G) -> None:
    n, seed = wl.n_weights, wl.seed
    for c0 in range(0, n, _CHUNK):
        cnt = min(_CHUNK, n - c0)
        # means: +-10^U(-6, 6)
        sign = torch.where(uniform(seed, STREAM_MU, c0, cnt, device, lane=0) < 0.5, -1.0, 1.0)
        m = sign * torch.pow(10.0, -6.0 + 12.0 * uniform(seed, STREAM_MU, c0, cnt, device, lane=1))
        # standard deviations: 89 % tiny, 10 % so small that sigma^2 underflows fp32,
        # 1 % within 1e-7..1e-3 of one (there the KL addends cancel and mu is tiny too)
        cat = uniform(seed, STREAM_SIGMA, c0, cnt, device, lane=0)
        u = uniform(seed, STREAM_SIGMA, c0, cnt, device, lane=1)
        tiny = torch.pow(10.0, -6.0 + 3.0 * u)
        under = torch.pow(10.0, -20.0 + 14.0 * u)
        pm = torch.where(uniform(seed, STREAM_SIGMA, c0, cnt, device, lane=2) < 0.5, -1.0, 1.0)
        near1 = 1.0 + pm * torch.pow(10.0, -7.0 + 4.0 * u)
        sd = torch.where(cat < 0.89, tiny, torch.where(cat < 0.99, under, near1))
        m = torch.where(cat >= 0.99, sign * 1e-4 * (0.5 + u), m)
        mu[c0:c0 + cnt] = m.to(torch.float32)
        sigma[c0:c0 + cnt] = sd.to(torch.float32)

    def eps_fn(s, c0, cnt):
        # N(0, 1) with about 1e-4 of the entries forced to 0, +6 or -6
        k0 = s * n + c0
        z = normal(seed, STREAM_EPS, k0, cnt, device)
        sel = uniform(seed, STREAM_EPS, k0, cnt, device, lane=2)
        z = torch.where(sel < 1e-4 / 3, torch.zeros_like(z), z)
        z = torch.where((sel >= 1e-4 / 3) & (sel < 2e-4 / 3), torch.full_like(z, 6.0), z)
        z = torch.where((sel >= 2e-4 / 3) & (sel < 1e-4), torch.full_like(z, -6.0), z)
        return z

    def g_fn(s, c0, cnt):
        # heavy-tailed Student-t (2 degrees of freedom), one magnitude 10^U(-8, 4) per block
        # of 4096 weights, plus a large component common to all samples whose sign
        # alternates with s (so the sum over samples cancels).
        k0 = s * n + c0
        z = normal(seed, STREAM_G, k0, cnt, device)
        t2 = z / torch.sqrt(-torch.log(uniform(seed, STREAM_G, k0, cnt, device, lane=2)))
        col = torch.arange(c0, c0 + cnt, dtype=torch.int64, device=device)
        scale = torch.pow(10.0, -8.0 + 12.0 * _uniform(seed, STREAM_AUX, (col // 4096) * 4))
        common = 100.0 * scale * (0.5 + _uniform(seed, STREAM_AUX, col * 4 + 1))
        return scale * t2 + (1.0 if s % 2 == 0 else -1.0) * common

    _fill_rows(eps, n, eps_fn)
    _fill_rows(G, n, g_fn)


def make_inputs(wl: Workload, device="cpu", base_offset: int = 0) -> Dict[str, torch.Tensor]:
    """mu[N], sigma[N], eps[S_loc, ld], G[S_loc, ld] as fp32 torch tensors on ``device``.

    Padding columns N..ld-1 of eps and G hold NaN: the path must never read them.
    ``base_offset`` > 0 places every array ``base_offset`` floats past a 256-byte aligned
    allocation (the misaligned-base variant of the adversarial case); the 2-D arrays are
    then views with row pitch ld.
    """
    n, s, ld = wl.n_weights, wl.s_local, wl.ld

    def alloc1(count):
        buf = torch.empty(count + base_offset, dtype=torch.float32, device=device)
        return buf[base_offset:base_offset + count]

    mu, sigma = alloc1(n), alloc1(n)
    eps = alloc1(s * ld).view(s, ld)
    G = alloc1(s * ld).view(s, ld)
    if ld > n:
        eps[:, n:] = float("nan")
        G[:, n:] = float("nan")
    if wl.kind == "paper":
        _paper_values(wl, device, mu, sigma, eps, G)
    elif wl.kind == "adversarial":
        _adversarial_values(wl, device, mu, sigma, eps, G)
    else:
        raise ValueError(wl.kind)
    return {"mu": mu, "sigma": sigma, "eps": eps, "G": G}
