"""Counter-based synthetic values, bit-identical on the host and on the GPU.

Every value is a pure function of (key, element index): no state, no libm.
key is derived from a seed and a tuple of small integers / strings naming the
stream (job, worker, round, ...).  For element i:

    z  = splitmix64 finalizer of (key + (i + 1) * GAMMA)        (64-bit wrap)
    k  = z[0:16] + z[16:32] + z[32:48] + z[48:64]               (0 .. 262140)
    x  = float32(k - 131070) * float32(std * sqrt(3) / 65536)

The sum of four 16-bit uniforms is bell-shaped with standard deviation
65536 / sqrt(3) (to 1 part in 10^9), so x has standard deviation std; it stands
in for the N(0, std) values of the workload configurations.  Only integer ops,
one exact int -> float32 conversion and one float32 multiply are used, so torch
computes the same bits on any device.  splitmix64 is the public-domain mixer of
Steele, Lea and Flood ("Fast splittable pseudorandom number generators", 2014).
"""
from __future__ import annotations

import hashlib
import math
from typing import List, Sequence

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _mix(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, *ids) -> int:
    """64-bit key of the stream named by ids (ints or strings) under seed."""
    k = _mix(int(seed) + _GAMMA)
    for t in ids:
        if isinstance(t, str):
            t = int.from_bytes(hashlib.sha256(t.encode()).digest()[:8], "little")
        k = _mix((k + _GAMMA) ^ (int(t) & _M64))
    return k


def _raw(key: int, i: int) -> int:
    return _mix(key + (i + 1) * _GAMMA)


def draw_from(seed: int, label: str, n: int, choices: Sequence[int]) -> List[int]:
    """n independent picks from choices (host-side, pure Python)."""
    key = stream_key(seed, label)
    return [choices[(_raw(key, i) >> 33) % len(choices)] for i in range(n)]


def _s64(x: int) -> int:
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    return (z >> k) & ((1 << (64 - k)) - 1)


def scale_constant(std: float) -> np.float32:
    return np.float32(std * math.sqrt(3.0) / 65536.0)


@torch.no_grad()
def fill_normal_like(out: torch.Tensor, key: int, std: float, start: int = 0,
                     chunk: int = 1 << 24) -> torch.Tensor:
    """Fill the 1-D float32 tensor out (on any device) with elements
    start .. start+len(out)-1 of stream key, standard deviation std."""
    assert out.dtype == torch.float32 and out.dim() == 1
    dev = out.device
    c = torch.tensor(float(scale_constant(std)), dtype=torch.float32, device=dev)
    n = out.numel()
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        z = torch.arange(start + lo + 1, start + hi + 1, dtype=torch.int64, device=dev)
        z = z * _s64(_GAMMA) + _s64(key)
        z = (z ^ _lsr(z, 30)) * _s64(_C1)
        z = (z ^ _lsr(z, 27)) * _s64(_C2)
        z = z ^ _lsr(z, 31)
        k = (z & 0xFFFF) + ((z >> 16) & 0xFFFF) + ((z >> 32) & 0xFFFF) + ((z >> 48) & 0xFFFF)
        torch.mul((k - 131070).to(torch.float32), c, out=out[lo:hi])
    return out


def reference_value(key: int, i: int, std: float) -> np.float32:
    """Element i of stream key by big-integer arithmetic (slow; for checks)."""
    z = _raw(key, i)
    k = (z & 0xFFFF) + ((z >> 16) & 0xFFFF) + ((z >> 32) & 0xFFFF) + (z >> 48)
    return np.float32(np.float32(k - 131070) * scale_constant(std))
