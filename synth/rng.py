"""Counter-based pseudo-random numbers for the synthetic workloads.

Every draw is a pure function of (seed, stream, index), so any slice of any
array can be regenerated without state and both the CPU checker and the GPU
library are handed byte-identical inputs.  The mixer is the published
splitmix64 finaliser applied to a 64-bit counter built from the key.

This module holds no scheduling arithmetic: only random bits, uniform and
normal variates.
"""
import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLD = np.uint64(0x9E3779B97F4A7C15)

# stream identifiers (one independent sequence each)
STREAM_X_ON, STREAM_X_OFF = 0, 1
STREAM_W1, STREAM_B1, STREAM_W2, STREAM_B2, STREAM_W3, STREAM_B3 = 2, 3, 4, 5, 6, 7
STREAM_MIXTURE, STREAM_MATRIX, STREAM_MASK, STREAM_PERM, STREAM_TYPE, STREAM_SM = 8, 9, 10, 11, 12, 13
STREAM_SLOW = 14


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def bits64(seed, stream, count, offset=0):
    """`count` 64-bit words for counters offset .. offset+count-1."""
    with np.errstate(over="ignore"):
        key = _mix(np.uint64(seed) * _GOLD + np.uint64(stream) + np.uint64(1))
        idx = np.arange(offset, offset + count, dtype=np.uint64)
        return _mix(_mix(key + idx * _GOLD) ^ key)


def uniform24(seed, stream, count, offset=0):
    """Uniform in [0,1) on a 2^-24 grid, exact in float32."""
    top = (bits64(seed, stream, count, offset) >> np.uint64(40)).astype(np.float64)
    return (top / 16777216.0).astype(np.float32)


def uniform53(seed, stream, count, offset=0):
    """Uniform in (0,1) with 53 random bits, float64 (never exactly 0)."""
    top = (bits64(seed, stream, count, offset) >> np.uint64(11)).astype(np.float64)
    return (top + 0.5) / 9007199254740992.0


def normal(seed, stream, count, offset=0):
    """Standard normal variates (Box-Muller on two 53-bit uniforms), float64."""
    u1 = uniform53(seed, stream, count, 2 * offset)
    u2 = uniform53(seed, stream, count, 2 * offset + 2 * count + 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def integers(seed, stream, count, high, offset=0):
    """Integers in [0, high) (high < 2^31), int64."""
    top = bits64(seed, stream, count, offset) >> np.uint64(33)
    return ((top * np.uint64(high)) >> np.uint64(31)).astype(np.int64)
