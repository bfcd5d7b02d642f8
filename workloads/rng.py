"""Counter-based random numbers: value k of stream (seed, stream) depends only on
(seed, stream, k), so any slice of any input can be regenerated independently of
numpy's own generator implementations and of chunking.

The mixer is the published splitmix64 finaliser (Steele, Lea, Flood 2014) applied to
seed-offset counters.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_base(seed, stream):
    # Python ints, wrapped to 64 bits: two mixing rounds decorrelate nearby seeds/streams.
    s = (int(seed) * 0x9E3779B97F4A7C15 + 0x632BE59BD9B4E019) & _MASK64
    t = (int(stream) * 0xD1342543DE82EF95 + 0x2545F4914F6CDD1D) & _MASK64
    with np.errstate(over="ignore"):
        b = _mix(np.uint64(s) ^ _mix(np.uint64(t)))
    return np.uint64(b)


def splitmix64(seed, stream, start, count):
    """`count` 64-bit values: counters start..start+count-1 of stream (seed, stream)."""
    with np.errstate(over="ignore"):
        ctr = np.arange(start, start + count, dtype=np.uint64)
        z = _stream_base(seed, stream) + (ctr + np.uint64(1)) * _GOLDEN
        return _mix(z)


def uniform01(seed, stream, start, count):
    """float64 in [0, 1) with 53 random bits."""
    return (splitmix64(seed, stream, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def uniform_pm1(seed, stream, start, count):
    """float64 in [-1, 1)."""
    return 2.0 * uniform01(seed, stream, start, count) - 1.0


def normal01(seed, stream, start, count):
    """float64 standard normal (Box-Muller, one output per counter pair)."""
    u1 = uniform01(seed, stream, 2 * start, 2 * count)
    a = u1[0::2]
    b = u1[1::2]
    # 1 - a is in (0, 1], so the log is finite.
    return np.sqrt(-2.0 * np.log1p(-a)) * np.cos(2.0 * np.pi * b)
