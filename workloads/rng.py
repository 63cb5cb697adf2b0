"""Counter-based random numbers on 64-bit integers, in torch, identical on CPU and GPU.

Everything here is integer arithmetic on int64 tensors (two's-complement wrap-around is
the same as unsigned arithmetic mod 2**64), so a workload generated on the CPU for a small
test and one generated on the GPU for a full-size run are the same function of
(seed, stream, index).  No floating point is used on the device: probability tables
(Zipf) are built once on the host as integer thresholds.

The mixer is the splitmix64 output function (Steele, Lea, Flood, "Fast splittable
pseudorandom number generators", OOPSLA 2014), a bijection of the 64-bit integers.
"""
from __future__ import annotations

import numpy as np
import torch

SEED = 0x5EED251116138

_M64 = (1 << 64) - 1


def _i64(x: int) -> int:
    """Python int (any sign) -> the int64 with the same low 64 bits."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _i64(0x9E3779B97F4A7C15)
_C1 = _i64(0xBF58476D1CE4E5B9)
_C2 = _i64(0x94D049BB133111EB)
_C3 = _i64(0xD6E8FEB86659FD93)


def lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical (zero-filling) right shift of an int64 tensor by 0 < s < 64."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def rotl(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x << s) | lsr(x, 64 - s)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser applied to x + golden-ratio increment.  Bijective."""
    z = x + _GOLDEN
    z = (z ^ lsr(z, 30)) * _C1
    z = (z ^ lsr(z, 27)) * _C2
    return z ^ lsr(z, 31)


def mix64_int(x: int) -> int:
    """Same function on one Python int (returned as unsigned 64-bit)."""
    z = (x + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """One 64-bit key per (seed, stream); streams name independent random sequences."""
    return _i64(mix64_int((mix64_int(seed & _M64) ^ (stream * 0xD6E8FEB86659FD93)) & _M64))


def u64(seed: int, stream: int, index: torch.Tensor) -> torch.Tensor:
    """Random 64 bits (as int64 bit patterns) for each counter value in `index`."""
    return mix64(index * _C3 ^ stream_key(seed, stream))


def below(seed: int, stream: int, index: torch.Tensor, n: int) -> torch.Tensor:
    """Integer in [0, n) from the top 31 bits of the counter's random word (n < 2**31).

    The modulo bias is below n / 2**31 and is part of the definition.
    """
    assert 0 < n < (1 << 31)
    return lsr(u64(seed, stream, index), 33) % n


def chance(seed: int, stream: int, index: torch.Tensor, p: float) -> torch.Tensor:
    """Bernoulli(p) as a bool tensor; the threshold is an integer fixed on the host."""
    thr = int(round(p * (1 << 31)))
    return lsr(u64(seed, stream, index), 33) < thr


def zipf_thresholds(n: int, a: float) -> np.ndarray:
    """Host-side integer CDF of a Zipf(a) law over ranks 1..n, scaled to 2**31."""
    w = 1.0 / np.power(np.arange(1, n + 1, dtype=np.float64), a)
    cdf = np.cumsum(w) / np.sum(w)
    thr = np.minimum(np.round(cdf * (1 << 31)).astype(np.int64), 1 << 31)
    thr[-1] = 1 << 31
    return thr


def zipf(seed: int, stream: int, index: torch.Tensor, thresholds: torch.Tensor) -> torch.Tensor:
    """Rank in [0, n) drawn from the integer CDF `thresholds` (on index's device)."""
    r = lsr(u64(seed, stream, index), 33)
    return torch.searchsorted(thresholds, r, right=True).clamp_(max=thresholds.numel() - 1)


def bswap64(x: torch.Tensor) -> torch.Tensor:
    """Reverse the byte order of each int64."""
    x = ((x & 0x00FF00FF00FF00FF) << 8) | (lsr(x, 8) & 0x00FF00FF00FF00FF)
    x = ((x & 0x0000FFFF0000FFFF) << 16) | (lsr(x, 16) & 0x0000FFFF0000FFFF)
    return (x << 32) | lsr(x, 32)


def ordered(x: torch.Tensor) -> torch.Tensor:
    """Map an unsigned 64-bit pattern to the int64 with the same order (flip the top bit)."""
    return x ^ _i64(1 << 63)
