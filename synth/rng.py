"""Counter-based seeded random numbers for the synthetic workloads.

Everything here is plain torch tensor arithmetic that gives the same bits on a
CPU tensor and on a device tensor: a 64-bit integer mixing function (the
splitmix64 finaliser, from its published definition) applied to a counter, and
a normal variate taken from a tabulated inverse normal CDF with linear
interpolation (gather + one subtract, one multiply, one add, each rounded
once).  No routing, caching or expert arithmetic lives in this package: it only
makes inputs, which are handed unchanged to both the CPU oracle and the HIP
library.
"""
from __future__ import annotations

import numpy as np
import torch

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Reinterpret an unsigned 64-bit constant as the signed value torch stores."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(v: torch.Tensor, n: int) -> torch.Tensor:
    """Logical right shift of int64 (torch's >> is arithmetic)."""
    return (v >> n) & ((1 << (64 - n)) - 1)


def mix64(v: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on an int64 tensor (wrapping arithmetic)."""
    v = (v ^ _lsr(v, 30)) * _M1
    v = (v ^ _lsr(v, 27)) * _M2
    return v ^ _lsr(v, 31)


def _mix64_int(v: int) -> int:
    v &= _MASK64
    v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _MASK64
    return v ^ (v >> 31)


def stream_key(seed: int, *ids: int) -> int:
    """Derive a 64-bit key for one named stream (seed plus integer ids)."""
    k = _mix64_int(seed * 0x9E3779B97F4A7C15 + 0x1234567)
    for i in ids:
        k = _mix64_int(k ^ ((int(i) + 1) * 0xD1B54A32D192ED03))
    return k


def random_bits(key: int, n: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """n 64-bit words of stream `key`, counters offset .. offset+n-1 (int64 tensor)."""
    ctr = torch.arange(offset, offset + n, dtype=torch.int64, device=device)
    return mix64(ctr * _GOLDEN + _s64(key))


_TABLE_BITS = 16
_table_cache: dict = {}


def _normal_table(device) -> torch.Tensor:
    dev = torch.device(device)
    tab = _table_cache.get(dev)
    if tab is None:
        from scipy.special import ndtri

        n = 1 << _TABLE_BITS
        p = np.arange(n + 1, dtype=np.float64) / n
        p = np.clip(p, 2.0 ** -(_TABLE_BITS + 1), 1.0 - 2.0 ** -(_TABLE_BITS + 1))
        tab = torch.from_numpy(ndtri(p).astype(np.float32)).to(dev)
        _table_cache[dev] = tab
    return tab


def standard_normal(key: int, n: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """n fp32 values ~ N(0,1) (|v| <= 4.33), identical on every device."""
    bits = random_bits(key, n, device, offset)
    idx = _lsr(bits, 64 - _TABLE_BITS)
    frac = (_lsr(bits, 64 - _TABLE_BITS - 16) & 0xFFFF).to(torch.float32) * (1.0 / 65536.0)
    tab = _normal_table(device)
    lo = tab[idx]
    hi = tab[idx + 1]
    return lo + frac * (hi - lo)


def uniform_ints(key: int, n: int, bound: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """n integers in [0, bound) (bound < 2**31), int64 tensor."""
    bits = _lsr(random_bits(key, n, device, offset), 33)  # 31 bits
    return (bits * bound) >> 31
