"""Seeded random streams for the synthetic layers.

This module only produces raw numbers (uniforms, normals, shuffles).  It holds
none of the method's arithmetic: no masking, no pattern assignment, no
convolution.  Both the CPU oracle and the HIP path consume the byte buffers made
here, so neither depends on the other.

Generator: SplitMix64 (Steele, Lea, Flood 2014), evaluated in counter form so a
whole tensor is produced by vectorised numpy: element i of stream `seed` is
mix(seed + (i + 1) * GOLDEN).
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1

BASE_SEED = 200107710


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def stream_seed(*parts: int) -> int:
    """Fold a tuple of small integers (config id, layer index, tensor kind, ...) into one 64-bit seed."""
    s = _mix_int(BASE_SEED)
    for p in parts:
        s = _mix_int(s ^ _mix_int((int(p) + 0x632BE59BD9B4E019) & _MASK64))
    return s


def raw_u64(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """n consecutive 64-bit outputs of the stream, starting at element `offset`."""
    with np.errstate(over="ignore"):
        idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        return _mix(np.uint64(seed & _MASK64) + idx * _GOLDEN)


def uniform01(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """Doubles in (0, 1]: (top 53 bits + 1) / 2**53, so that log() is always finite."""
    top = raw_u64(seed, n, offset) >> np.uint64(11)
    return (top.astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal(seed: int, n: int) -> np.ndarray:
    """n standard normals in double by Box-Muller; pair j uses uniforms 2j and 2j+1."""
    m = (n + 1) // 2
    u = uniform01(seed, 2 * m)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    t = (2.0 * np.pi) * u[1::2]
    out = np.empty(2 * m, dtype=np.float64)
    out[0::2] = r * np.cos(t)
    out[1::2] = r * np.sin(t)
    return out[:n]


def randint(seed: int, n: int, hi: int) -> np.ndarray:
    """n integers in [0, hi) (hi << 2**64, so the modulo bias is far below anything a test could see)."""
    return (raw_u64(seed, n) % np.uint64(hi)).astype(np.int64)


def shuffle(seed: int, items: list) -> list:
    """Fisher-Yates shuffle of a copy of `items`, drawing from the stream in order."""
    a = list(items)
    draws = raw_u64(seed, max(len(a) - 1, 0))
    k = 0
    for i in range(len(a) - 1, 0, -1):
        j = int(draws[k]) % (i + 1)
        k += 1
        a[i], a[j] = a[j], a[i]
    return a
