"""Seeded synthetic input generators shared by the CPU oracle and the HIP path.

This module holds no arithmetic of the training method: only a counter-based
random number generator and the distributions the workloads draw from
(standard normal pixels / sensor windows, uniform labels, normal weight
initialisation with a caller-given standard deviation, uniform reals for
device capacities).  Every value is a pure function of (seed, stream name,
element index), so both sides receive exactly the same arrays regardless of
the order in which they ask for them.

Generator: element i of stream s under seed k is
    mix64(key + (i + 1) * GOLDEN),  key = mix64(mix64(k) ^ fnv1a64(s))
with mix64 the SplitMix64 output function.  Uniforms take the top 53 bits;
normals use the Box-Muller transform on two consecutive counters.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _fnv1a64(name):
    h = 0xCBF29CE484222325
    for b in name.encode("utf-8"):
        h = ((h ^ b) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return np.uint64(h)


def bits(seed, stream, n, offset=0):
    """n raw 64-bit words of the stream, starting at counter `offset`."""
    key = _mix64(_mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF)) ^ _fnv1a64(stream))
    ctr = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(key + ctr * _GOLDEN)


def uniform01(seed, stream, n, offset=0):
    """n doubles uniform in [0, 1)."""
    return (bits(seed, stream, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def uniform(seed, stream, shape, lo=0.0, hi=1.0):
    n = int(np.prod(shape))
    return (lo + (hi - lo) * uniform01(seed, stream, n)).reshape(shape)


def normal(seed, stream, shape, std=1.0, chunk=1 << 22):
    """Standard normal (times std), float64, one Box-Muller draw per element."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float64)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        u = uniform01(seed, stream, 2 * m, offset=2 * s)
        r = np.sqrt(-2.0 * np.log1p(-u[0::2]))          # 1-u in (0,1]
        out[s:s + m] = r * np.cos(2.0 * np.pi * u[1::2])
    if std != 1.0:
        out *= std
    return out.reshape(shape)


def labels(seed, stream, n, classes):
    """n int32 labels uniform in 0..classes-1."""
    return (bits(seed, stream, n) % np.uint64(classes)).astype(np.int32)


def integers(seed, stream, shape, lo, hi):
    """Integers uniform in lo..hi inclusive, as float64 (exactly representable)."""
    n = int(np.prod(shape))
    return (lo + (bits(seed, stream, n) % np.uint64(hi - lo + 1)).astype(np.float64)).reshape(shape)
