"""Seeded synthetic values: identical bits on CPU and GPU, no libm.

Every value is a pure function of (seed, step, stream, flat element index):

    x   = (index + stream_key(seed, step, stream))            mod 2^64
    z   = splitmix64 finaliser of x                            (integer)
    s   = sum of z's four 16-bit fields - 131070               (|s| < 2^18, Irwin-Hall)
    val = fp32(s) * scale[tensor holding index]                (one IEEE multiply)

``fp32(s)`` is exact, and the single multiply rounds the same way everywhere,
so torch on the CPU, torch on the GPU and the numpy twin in the tests all
produce the same bits.  s is approximately normal with standard deviation
STD_S, so ``scale = sigma / STD_S`` gives values of standard deviation sigma.

This module is input generation only.  It holds none of the arithmetic of the
method under test and is the only code both the CPU oracle's tests and the GPU
path's tests draw on.
"""
from __future__ import annotations

from math import sqrt
from typing import Optional

import torch

from .buckets import Layout

MASK64 = (1 << 64) - 1
STD_S = sqrt(4 * ((1 << 32) - 1) / 12.0)       # std of the sum of four uniform 16-bit ints

# stream ids: ESTs use their virtual rank; other streams sit far above any rank
STREAM_PARAM = 1 << 20
STREAM_BN = 1 << 21


def _splitmix_int(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & MASK64
    return x ^ (x >> 31)


def stream_key(seed: int, step: int, stream: int) -> int:
    k = _splitmix_int(seed & MASK64)
    k = _splitmix_int(k ^ (step & MASK64))
    k = _splitmix_int(k ^ ((stream * 0x100000001B3) & MASK64))
    return k


def _s64(x: int) -> int:
    """Reinterpret an unsigned 64-bit value as the signed value with the same bits."""
    x &= MASK64
    return x - (1 << 64) if x >> 63 else x


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    return (z >> k) & ((1 << (64 - k)) - 1)


def field_sums(lo: int, hi: int, key: int, device="cpu") -> torch.Tensor:
    """int64 tensor of s for flat indices [lo, hi)."""
    x = torch.arange(lo, hi, dtype=torch.int64, device=device) + _s64(key)
    z = x + _s64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    z = z ^ _lsr(z, 31)
    s = (z & 0xFFFF) + (_lsr(z, 16) & 0xFFFF) + (_lsr(z, 32) & 0xFFFF) + (_lsr(z, 48) & 0xFFFF)
    return s - 131070


def field_sums_at(idx: torch.Tensor, key: int) -> torch.Tensor:
    """int64 tensor of s for an arbitrary int64 tensor of flat indices."""
    x = idx + _s64(key)
    z = x + _s64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    z = z ^ _lsr(z, 31)
    s = (z & 0xFFFF) + (_lsr(z, 16) & 0xFFFF) + (_lsr(z, 32) & 0xFFFF) + (_lsr(z, 48) & 0xFFFF)
    return s - 131070


def scales_at(layout: Layout, idx: torch.Tensor, sigma0: float, use_fan_in: bool) -> torch.Tensor:
    """fp32 per-element scale for arbitrary flat indices (same values as ``scales``)."""
    starts = torch.tensor([off for off, _, _ in layout.tensors], dtype=torch.int64, device=idx.device)
    vals = torch.tensor([(sigma0 / sqrt(f) if use_fan_in else sigma0) / STD_S for _, _, f in layout.tensors],
                        dtype=torch.float32, device=idx.device)
    which = torch.searchsorted(starts, idx, right=True) - 1
    return vals[which]


def values_at(layout: Layout, idx: torch.Tensor, seed: int, step: int, stream: int,
              sigma0: float = 1e-2, use_fan_in: bool = True) -> torch.Tensor:
    """fp32 synthetic values at arbitrary flat indices; same bits as ``values`` on ranges."""
    s = field_sums_at(idx, stream_key(seed, step, stream)).to(torch.float32)
    return s * scales_at(layout, idx, sigma0, use_fan_in)


def scales(layout: Layout, lo: int, hi: int, sigma0: float, use_fan_in: bool,
           device="cpu") -> torch.Tensor:
    """fp32 per-element scale for flat indices [lo, hi): sigma0 / sqrt(fan_in) / STD_S."""
    vals, reps = [], []
    for off, ln, fan_in in layout.tensors:
        a, b = max(off, lo), min(off + ln, hi)
        if a < b:
            sigma = sigma0 / sqrt(fan_in) if use_fan_in else sigma0
            vals.append(sigma / STD_S)
            reps.append(b - a)
    v = torch.tensor(vals, dtype=torch.float32, device=device)
    r = torch.tensor(reps, dtype=torch.int64, device=device)
    return torch.repeat_interleave(v, r)


def values(layout: Layout, lo: int, hi: int, seed: int, step: int, stream: int,
           sigma0: float = 1e-2, use_fan_in: bool = True, device="cpu",
           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """fp32 synthetic values for flat indices [lo, hi) of ``layout``."""
    if hi <= lo:
        return torch.empty(0, dtype=torch.float32, device=device)
    s = field_sums(lo, hi, stream_key(seed, step, stream), device).to(torch.float32)
    res = torch.mul(s, scales(layout, lo, hi, sigma0, use_fan_in, device), out=out)
    return res


def gradient(layout: Layout, bucket: int, seed: int, step: int, est: int,
             device="cpu", out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Gradient bucket ``bucket`` of logical worker ``est`` at global step ``step``."""
    off, ln = layout.buckets[bucket]
    return values(layout, off, off + ln, seed, step, est, 1e-2, True, device, out)


def params(layout: Layout, seed: int, device="cpu") -> torch.Tensor:
    """Initial parameter vector p0 (sigma = 1/sqrt(fan_in))."""
    return values(layout, 0, layout.n_params, seed, 0, STREAM_PARAM, 1.0, True, device)


def small_ints(n: int, seed: int, step: int, stream: int, span: int = 8,
               device="cpu") -> torch.Tensor:
    """Integer-valued fp32 in [-span, span): sums of these are exact in any order."""
    s = field_sums(0, n, stream_key(seed, step, stream), device)
    return (torch.remainder(s, 2 * span) - span).to(torch.float32)
