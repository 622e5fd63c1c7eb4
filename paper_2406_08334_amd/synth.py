"""Seeded, counter-based synthetic inputs for model states.

The value of element `e` depends only on (seed, step, stream, e): it does not
depend on how the range is split into calls, tensors or chunks, nor on the
device the generator runs on up to the last bit of the library's log/cos (one
call produces the bytes once; every consumer is handed those same bytes).

This module holds none of the method's arithmetic: an integer hash (the
splitmix64 finaliser), Box-Muller in fp64, a scale, and the library's own
round-to-nearest conversion to the 16-bit storage type.
"""
from __future__ import annotations

import math

import torch

SEED_PARAMS = 0x5EED0001
SEED_GRADS = 0x5EED0002
SEED_INF = 0x5EED0003

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_BLOCK = 1 << 24


def _s64(x: int) -> int:
    """Python int -> the int64 value with the same low 64 bits."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_int(x: int) -> int:
    x &= _M64
    x ^= x >> 30
    x = (x * _C1) & _M64
    x ^= x >> 27
    x = (x * _C2) & _M64
    x ^= x >> 31
    return x


def stream_key(seed: int, step: int, stream: int) -> int:
    return _mix_int(_mix_int(_mix_int(seed) ^ (step * _GOLDEN)) ^ (stream * _C1))


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = x ^ _lsr(x, 30)
    x = x * _s64(_C1)
    x = x ^ _lsr(x, 27)
    x = x * _s64(_C2)
    x = x ^ _lsr(x, 31)
    return x


def hash_u64(key: int, start: int, count: int, device) -> torch.Tensor:
    """int64 tensor holding hash(key, e) for e in [start, start+count)."""
    e = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix((e * _s64(_GOLDEN)) ^ _s64(key))


def standard_normal(key: int, start: int, count: int, device) -> torch.Tensor:
    """fp64 N(0,1) draws for elements [start, start+count)."""
    z1 = hash_u64(key, start, count, device)
    z2 = _mix(z1 ^ _s64(0xD1B54A32D192ED03))
    u1 = (_lsr(z1, 11) + 1).to(torch.float64) * (2.0 ** -53)      # (0, 1]
    u2 = _lsr(z2, 11).to(torch.float64) * (2.0 ** -53)            # [0, 1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def normal_16(seed: int, step: int, stream: int, start: int, count: int, std: float,
              dtype: torch.dtype, device, scale: float = 1.0, outlier_every: int = 0,
              outlier_gain: float = 100.0, out: torch.Tensor | None = None) -> torch.Tensor:
    """N(0, std) draws, as fp32, times `scale`, rounded by torch to bf16/fp16.

    outlier_every > 0: element e is multiplied by outlier_gain (before rounding)
    iff hash(key', e) mod outlier_every == 0.
    """
    assert dtype in (torch.bfloat16, torch.float16)
    key = stream_key(seed, step, stream)
    if out is None:
        out = torch.empty(count, dtype=dtype, device=device)
    assert out.numel() == count
    for lo in range(0, count, _BLOCK):
        n = min(_BLOCK, count - lo)
        x = (standard_normal(key, start + lo, n, device) * std).to(torch.float32)
        if outlier_every > 0:
            hz = hash_u64(_mix_int(key ^ 0xA5A5A5A5), start + lo, n, device)
            pick = torch.remainder(_lsr(hz, 1), outlier_every) == 0
            x = torch.where(pick, x * outlier_gain, x)
        if scale != 1.0:
            x = x * scale
        out[lo:lo + n] = x.to(dtype)
    return out


def pick_element(seed: int, step: int, n_real: int) -> int:
    """A seeded global element index in [0, n_real) (used to plant one +inf)."""
    return _mix_int(stream_key(seed, step, 0)) % n_real


def as_u16(t: torch.Tensor):
    """numpy uint16 view of a CPU bf16/fp16 tensor's bits."""
    import numpy as np
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)
