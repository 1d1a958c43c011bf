"""Seeded input pools and arrival traces."""
import numpy as np

from . import rng
from .blob import DT_I8, f32_to_bf16_bits
from .nets import BASE_SEED

_POOL_STREAM = 0x1000
_TRACE_STREAM = 0x2000


def input_pool(blob, n, seed_off=0, first=0):
    """Samples first..first+n-1 of the pool for `blob`: [n][H][W][C].

    int8 networks: int8 uniform over [-128, 127]; bf16 networks: N(0,1) rounded to
    bf16 (returned as uint16 bit patterns).  Sample k depends only on (seed, k).
    """
    h, w, c = blob.in_shape()
    per = h * w * c
    seed = BASE_SEED + 0x100 + seed_off
    if blob.dtype == DT_I8:
        assert per % 8 == 0
        raw = rng.uniform_bytes(seed, _POOL_STREAM, n * per, start_word=first * per // 8)
        return raw.view(np.int8).reshape(n, h, w, c)
    out = np.empty((n, per), np.uint16)
    for i in range(n):   # one stream per sample keeps any slice reproducible
        out[i] = f32_to_bf16_bits(rng.normal_f64(seed, _POOL_STREAM + 1 + first + i, per).astype(np.float32))
    return out.reshape(n, h, w, c)


def poisson_trace(n, rate_per_s, seed_off=0):
    """Arrival times (int64 ns, non-decreasing, first at 0) of a Poisson process of the given rate."""
    u = rng.uniform_u01(BASE_SEED + 0x200 + seed_off, _TRACE_STREAM, n)
    gaps = -np.log(u) / float(rate_per_s)
    gaps[0] = 0.0
    return np.floor(np.cumsum(gaps) * 1e9).astype(np.int64)


def spiky_trace(n, rate_per_s, seed_off=0, period=5000, spike_start=4000, spike_len=1000, factor=5.0):
    """Poisson arrivals whose rate is multiplied by `factor` for requests
    [period*k + spike_start, period*k + spike_start + spike_len)."""
    u = rng.uniform_u01(BASE_SEED + 0x300 + seed_off, _TRACE_STREAM, n)
    idx = np.arange(n) % period
    rate = np.where((idx >= spike_start) & (idx < spike_start + spike_len), factor * rate_per_s, rate_per_s)
    gaps = -np.log(u) / rate
    gaps[0] = 0.0
    return np.floor(np.cumsum(gaps) * 1e9).astype(np.int64)
