"""Counter-based random numbers: value = mix(seed, stream, counter).

Every draw is a pure function of (seed, stream, counter), so any consumer can
regenerate exactly the same bytes without shared state.  The mixer is the
64-bit finaliser of the SplitMix64 generator (Steele, Lea, Flood 2014) applied
to seed, stream and counter combined with odd multipliers.
"""
import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_STREAM_MUL = np.uint64(0xD1342543DE82EF95)


def _mix64(z):
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def bits64(seed, stream, n, offset=0):
    """n 64-bit words for counters offset .. offset+n-1."""
    with np.errstate(over="ignore"):
        ctr = np.arange(offset, offset + n, dtype=np.uint64)
        base = _mix64(np.array([np.uint64(seed) * _GOLD + np.uint64(stream) * _STREAM_MUL + np.uint64(1)],
                               dtype=np.uint64))[0]
        return _mix64(ctr * _GOLD + base)


def uniform01(seed, stream, n, offset=0):
    """float64 in the open interval (0, 1), 53 random bits."""
    b = bits64(seed, stream, n, offset)
    return ((b >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed, stream, n):
    """Standard normal float64 by the Box-Muller transform (cosine branch)."""
    u1 = uniform01(seed, stream, n, 0)
    u2 = uniform01(seed, stream, n, 1 << 40)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def randint(seed, stream, n, hi):
    """Integers uniform on [0, hi)."""
    return np.minimum((uniform01(seed, stream, n) * hi).astype(np.int64), hi - 1)
