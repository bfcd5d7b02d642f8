"""Seeded feature matrices.  Values are float32; for bf16 workloads they are rounded once
(round-to-nearest-even) so that the float32 array holds exactly bf16-representable values:
the oracle reads that float32 array, the GPU library reads the matching 16-bit patterns."""
import numpy as np

from .rng import uniform_pm1, normal01

_CHUNK = 1 << 22


def _fill(fn, n, d, seed, stream):
    out = np.empty(n * d, dtype=np.float32)
    for s in range(0, n * d, _CHUNK):
        c = min(_CHUNK, n * d - s)
        out[s:s + c] = fn(seed, stream, s, c)
    return out.reshape(n, d)


def features_uniform(n, d, seed, stream=101):
    """float32 n x d, uniform in [-1, 1)."""
    return _fill(uniform_pm1, n, d, seed, stream)


def features_normal(n, d, seed, stream=102):
    """float32 n x d, standard normal."""
    return _fill(normal01, n, d, seed, stream)


def bf16_bits(x):
    """uint16 bit patterns of float32 `x` rounded to bfloat16 (nearest, ties to even).
    Inputs are finite by construction."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def round_to_bf16(x):
    """float32 array whose values are exactly the bf16 roundings of `x`."""
    return (bf16_bits(x).astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(np.shape(x))
