"""Counter-based random numbers: splitmix64 of (seed, stream, index).

Every tensor is a pure function of (seed, stream id, element index), so any
slice can be regenerated on any machine without state.
"""
import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLD = np.uint64(0x9E3779B97F4A7C15)


def splitmix64(x):
    """The splitmix64 output function applied to an array of uint64 counters."""
    with np.errstate(over="ignore"):
        z = (np.asarray(x, dtype=np.uint64) + _GOLD)
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _counters(seed, stream, start, count):
    with np.errstate(over="ignore"):
        base = splitmix64(np.uint64(seed) ^ (np.uint64(stream) * _M2))
        return base + np.arange(start, start + count, dtype=np.uint64)


def raw_u64(seed, stream, count, start=0):
    return splitmix64(_counters(seed, stream, start, count))


def uniform_bytes(seed, stream, count, start_word=0):
    """`count` bytes, uniform over 0..255 (8 per 64-bit draw)."""
    words = (count + 7) // 8
    out = np.empty(words * 8, dtype=np.uint8)
    step = 1 << 24
    for w0 in range(0, words, step):
        w1 = min(words, w0 + step)
        out[w0 * 8:w1 * 8] = raw_u64(seed, stream, w1 - w0, start_word + w0).view(np.uint8)
    return out[:count]


def uniform_u01(seed, stream, count, start=0):
    """float64 uniform on (0, 1): 53 random bits, never exactly 0."""
    r = raw_u64(seed, stream, count, start) >> np.uint64(11)
    return (r.astype(np.float64) + 0.5) * (1.0 / (1 << 53))


def normal_f64(seed, stream, count):
    """Standard normal float64 by Box-Muller on two uniform streams."""
    half = (count + 1) // 2
    out = np.empty(half * 2, dtype=np.float64)
    step = 1 << 22
    for h0 in range(0, half, step):
        h1 = min(half, h0 + step)
        u = uniform_u01(seed, stream, 2 * (h1 - h0), 2 * h0)
        rad = np.sqrt(-2.0 * np.log(u[0::2]))
        ang = 2.0 * np.pi * u[1::2]
        out[2 * h0:2 * h1:2] = rad * np.cos(ang)
        out[2 * h0 + 1:2 * h1:2] = rad * np.sin(ang)
    return out[:count]
