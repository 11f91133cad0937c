"""Counter-based seeded random numbers for the synthetic inputs.

Every value is a pure function of (seed, stream, index), so any slice of any
tensor can be regenerated without generating what precedes it, and the result
does not depend on numpy's own generators or on the order of calls.

The 64-bit mixer is the SplitMix64 finaliser (Steele, Lea, Flood 2014); normals
come from the Box-Muller transform of two uniforms.  This module holds no
detector arithmetic: it only produces input data.
"""
import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _stream_key(seed, stream):
    with np.errstate(over="ignore"):
        s = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + _GOLD * np.uint64((stream + 1) & 0xFFFFFFFFFFFFFFFF)
    return _mix64(s)


def bits64(seed, stream, start, count):
    """uint64[count]: raw bits for indices start .. start+count-1 of a stream."""
    key = _stream_key(seed, stream)
    idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(key + _GOLD * idx)


def uniform(seed, stream, count, start=0):
    """float64[count] in [0, 1)."""
    return (bits64(seed, stream, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal(seed, stream, count, start=0):
    """float64[count], standard normal; value i uses uniforms 2i and 2i+1."""
    u = uniform(seed, stream, 2 * count, 2 * start)
    u1 = 1.0 - u[0::2]          # (0, 1]
    u2 = u[1::2]
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def randint(seed, stream, lo, hi, count, start=0):
    """int64[count] uniform on lo..hi inclusive."""
    u = uniform(seed, stream, count, start)
    return lo + np.minimum((u * (hi - lo + 1)).astype(np.int64), hi - lo)
