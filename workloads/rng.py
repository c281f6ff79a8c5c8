"""Counter-based seeded random streams for the synthetic workloads.

This module only draws random numbers.  It holds none of the protocol's
arithmetic (no fixed-point encoding, no share splitting, no Beaver algebra):
the CPU oracle and the HIP path both consume the raw streams produced here.

Every stream is addressed by ``(seed, stream_id)`` and is random access:
element ``i`` depends on ``(seed, stream_id, i)`` only, so any slice can be
regenerated on any host.  The bit mixer is the public splitmix64 finaliser
(Steele, Lea, Flood 2014; Vigna's public-domain formulation).
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20250507

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _stream_key(seed: int, stream_id: int) -> np.uint64:
    k = (seed * 0x9E3779B97F4A7C15 + stream_id * 0xBF58476D1CE4E5B9 + 0x632BE59BD9B4E019) & _MASK64
    return _mix64(np.array([k], dtype=np.uint64))[0]


def uniform_u64(seed: int, stream_id: int, n: int, offset: int = 0) -> np.ndarray:
    """``n`` uniform 64-bit words, elements ``offset .. offset+n`` of the stream."""
    key = _stream_key(seed, stream_id)
    out = np.empty(n, dtype=np.uint64)
    chunk = 1 << 22
    with np.errstate(over="ignore"):
        for s in range(0, n, chunk):
            e = min(n, s + chunk)
            ctr = np.arange(offset + s + 1, offset + e + 1, dtype=np.uint64)
            out[s:e] = _mix64(key + ctr * _GOLDEN)
    return out


def uniform_01(seed: int, stream_id: int, n: int, offset: int = 0) -> np.ndarray:
    """``n`` float64 values in the open interval (0, 1) (53 random bits each)."""
    u = uniform_u64(seed, stream_id, n, offset)
    return ((u >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def gaussian_f64(seed: int, stream_id: int, n: int) -> np.ndarray:
    """``n`` standard normal float64 values (Box-Muller on two uniform streams)."""
    half = (n + 1) // 2
    u1 = uniform_01(seed, stream_id, half, 0)
    u2 = uniform_01(seed, stream_id, half, 1 << 40)
    r = np.sqrt(-2.0 * np.log(u1))
    t = 2.0 * np.pi * u2
    out = np.empty(2 * half, dtype=np.float64)
    out[0::2] = r * np.cos(t)
    out[1::2] = r * np.sin(t)
    return out[:n]


# ---------------------------------------------------------------------------
# the same streams drawn on a torch device (plumbing for large device-resident inputs)
# ---------------------------------------------------------------------------

def _s64(c: int) -> int:
    """A 64-bit constant as the signed value with the same bits (torch has no uint64 arithmetic)."""
    c &= _MASK64
    return c - (1 << 64) if c >= (1 << 63) else c


def uniform_u64_torch(seed: int, stream_id: int, n: int, device, offset: int = 0):
    """Elements ``offset .. offset+n`` of stream ``(seed, stream_id)`` as an ``int64`` torch
    tensor on ``device`` whose bits equal :func:`uniform_u64` word for word (two's-complement
    wrap-around multiplication, logical shifts emulated by masking)."""
    import torch
    key = _s64(int(_stream_key(seed, stream_id)))
    out = torch.empty(n, dtype=torch.int64, device=device)
    chunk = 1 << 26

    def lsr(z, s):
        return (z >> s) & ((1 << (64 - s)) - 1)

    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        z = torch.arange(offset + s + 1, offset + e + 1, dtype=torch.int64, device=device)
        z = z * _s64(int(_GOLDEN)) + key
        z = (z ^ lsr(z, 30)) * _s64(int(_M1))
        z = (z ^ lsr(z, 27)) * _s64(int(_M2))
        out[s:e] = z ^ lsr(z, 31)
    return out
