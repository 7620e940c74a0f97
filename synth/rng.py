"""Counter-based seeded generator with bit-identical numpy (host) and torch (host or device) back ends.

value(seed, stream, index) depends only on its three integer arguments, so any slice of any tensor
can be regenerated alone, on the host for a checker or on the GPU for bulk fills, with the same bits.

Recipe (all steps are integer operations or single, separately rounded IEEE fp32 operations, which
is what makes the two back ends agree bit for bit):
  h   = mix64(index + key(seed, stream))                 64-bit avalanche hash (splitmix-style)
  i   = top 16 bits of h, f = next 24 bits of h
  z   = Q[i] + D[i] * (f * 2^-24)                        piecewise-linear inverse normal CDF,
                                                         Q = 65537 quantile knots (fp32), D = Q[i+1]-Q[i]
  x   = z * sigma                                        fp32
  bf16 outputs keep the upper 16 bits of x (truncation; an input-generation choice, not a cast the
  method defines).
The distribution is a standard normal truncated at about +-4.3 sigma.
"""
from __future__ import annotations

import functools

import numpy as np

_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_K1 = 0x9E3779B97F4A7C15
_K2 = 0xD1B54A32D192ED03
_MASK64 = (1 << 64) - 1
_N_KNOTS = 65537


def _key(seed: int, stream: int) -> int:
    return ((seed & _MASK64) * _K1 + (stream & _MASK64) * _K2 + 0x632BE59BD9B4E019) & _MASK64


def _s64(x: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit constant."""
    return x - (1 << 64) if x >= (1 << 63) else x


@functools.lru_cache(maxsize=None)
def _tables_np():
    from scipy.special import ndtri
    k = np.arange(_N_KNOTS, dtype=np.float64)
    q = ndtri((k + 0.5) / _N_KNOTS).astype(np.float32)
    d = (q[1:] - q[:-1]).astype(np.float32)
    return q[:-1].copy(), d


@functools.lru_cache(maxsize=None)
def _tables_torch(device: str):
    import torch
    q, d = _tables_np()
    return torch.from_numpy(q).to(device), torch.from_numpy(d).to(device)


def hash64_np(seed: int, stream: int, start: int, n: int) -> np.ndarray:
    """uint64 hash of indices start..start+n-1 (numpy back end)."""
    with np.errstate(over="ignore"):
        x = np.arange(n, dtype=np.uint64) + np.uint64((start + _key(seed, stream)) & _MASK64)
        x ^= x >> np.uint64(30)
        x *= np.uint64(_M1)
        x ^= x >> np.uint64(27)
        x *= np.uint64(_M2)
        x ^= x >> np.uint64(31)
    return x


def _normal_np(seed, stream, start, n, sigma):
    h = hash64_np(seed, stream, start, n)
    q, d = _tables_np()
    i = (h >> np.uint64(48)).astype(np.int64)
    f = ((h >> np.uint64(24)) & np.uint64(0xFFFFFF)).astype(np.float32)
    t = f * np.float32(2.0 ** -24)
    z = q[i] + d[i] * t
    return (z * np.float32(sigma)).astype(np.float32, copy=False)


def _lsr(x, s):
    """Logical shift right of a torch int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _normal_torch(seed, stream, start, n, sigma, device):
    import torch
    dev = str(device)
    q, d = _tables_torch(dev)
    x = torch.arange(n, dtype=torch.int64, device=dev) + _s64((start + _key(seed, stream)) & _MASK64)
    x = x ^ _lsr(x, 30)
    x = x * _s64(_M1)
    x = x ^ _lsr(x, 27)
    x = x * _s64(_M2)
    x = x ^ _lsr(x, 31)
    i = _lsr(x, 48)
    f = (_lsr(x, 24) & 0xFFFFFF).to(torch.float32)
    del x
    t = f * (2.0 ** -24)
    z = d[i] * t
    z = q[i] + z
    return z * float(np.float32(sigma))


def normal_f32(seed: int, stream: int, start: int, n: int, sigma: float, device=None):
    """n fp32 values ~ N(0, sigma) for element indices start.. of the given stream.

    device=None returns a numpy array; otherwise a torch tensor on that device ("cpu", "cuda:0").
    """
    if device is None:
        return _normal_np(seed, stream, start, n, sigma)
    return _normal_torch(seed, stream, start, n, sigma, device)


def normal_bf16(seed: int, stream: int, start: int, n: int, sigma: float, device=None):
    """Same values truncated to bf16.  numpy: uint16 bit patterns; torch: a bfloat16 tensor."""
    x = normal_f32(seed, stream, start, n, sigma, device)
    if device is None:
        return x.view(np.uint16)[1::2].copy()
    import torch
    return x.view(torch.int16)[1::2].contiguous().view(torch.bfloat16)
