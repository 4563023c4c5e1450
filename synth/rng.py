"""Counter-based seeded random numbers for the synthetic workloads.

Every tensor of a workload is a pure function of (seed, tensor name, element
index): value i of a stream is a SplitMix64 finaliser applied to a counter, so
any slice can be regenerated on its own, in any order, on any machine.  This
module only draws numbers; it contains nothing of the sparsification method.
"""
from __future__ import annotations

import hashlib

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def _mix(z: np.ndarray) -> np.ndarray:
    """SplitMix64 output function on a uint64 array (wrapping arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def stream_base(seed: int, name: str) -> int:
    """Start of the sub-stream for one named tensor of one seeded workload."""
    h = hashlib.sha256(f"{seed & _MASK64:016x}/{name}".encode()).digest()
    return int.from_bytes(h[:8], "little")


def raw_u64(seed: int, name: str, start: int, count: int) -> np.ndarray:
    """Elements [start, start+count) of the uint64 stream (seed, name)."""
    base = stream_base(seed, name)
    with np.errstate(over="ignore"):
        ctr = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix(np.uint64(base) + ctr * _GAMMA)


def uniform01(seed: int, name: str, start: int, count: int) -> np.ndarray:
    """float64 uniforms in (0, 1], 53 bits each."""
    r = raw_u64(seed, name, start, count) >> np.uint64(11)
    return (r.astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def uniform(seed: int, name: str, shape, lo: float, hi: float) -> np.ndarray:
    n = int(np.prod(shape))
    u = uniform01(seed, name, 0, n)
    return (lo + (hi - lo) * u).reshape(shape)


def normal(seed: int, name: str, shape, chunk: int = 1 << 22) -> np.ndarray:
    """Standard normals (Box-Muller on pairs of the uniform stream), float32.

    Element 2j and 2j+1 come from uniforms 2j, 2j+1, so the result does not
    depend on the chunking.
    """
    n = int(np.prod(shape))
    out = np.empty(n + (n & 1), dtype=np.float32)
    pairs = out.size // 2
    step = chunk // 2
    for p0 in range(0, pairs, step):
        p1 = min(pairs, p0 + step)
        u = uniform01(seed, name, 2 * p0, 2 * (p1 - p0)).reshape(-1, 2)
        r = np.sqrt(-2.0 * np.log(u[:, 0]))
        th = (2.0 * np.pi) * u[:, 1]
        out[2 * p0:2 * p1:2] = r * np.cos(th)
        out[2 * p0 + 1:2 * p1:2] = r * np.sin(th)
    return out[:n].reshape(shape)


def permutation(seed: int, name: str, n: int) -> np.ndarray:
    """A seeded permutation of range(n): argsort of n stream values."""
    keys = raw_u64(seed, name, 0, n)
    return np.argsort(keys, kind="stable").astype(np.int32)


def bernoulli(seed: int, name: str, shape, p: float) -> np.ndarray:
    n = int(np.prod(shape))
    return (uniform01(seed, name, 0, n) <= p).astype(np.uint8).reshape(shape)
