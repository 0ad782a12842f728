"""Counter-based random numbers for the synthetic inputs.

Every draw is a pure function of (key, counter), so any element of any input
can be regenerated anywhere (host or device) without holding state or tables.
This module holds no arithmetic of the method under test: it only makes inputs.

The mixer is the published SplitMix64 output function (Steele, Lea, Flood:
"Fast splittable pseudorandom number generators", OOPSLA 2014): the state is
advanced by the odd constant GAMMA and finalised by two multiply/xor-shift
rounds.
"""
import numpy as np

GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_S30, _S27, _S31, _S11 = np.uint64(30), np.uint64(27), np.uint64(31), np.uint64(11)
_ONE = np.uint64(1)


def mix64(x):
    """SplitMix64 finaliser on an array (or scalar) of uint64, wrapping mod 2**64."""
    with np.errstate(over="ignore"):
        x = np.asarray(x, dtype=np.uint64)
        x = (x ^ (x >> _S30)) * _M1
        x = (x ^ (x >> _S27)) * _M2
        return x ^ (x >> _S31)


def u64(key, ctr):
    """The ctr-th 64-bit word of stream `key`: mix64(key + (ctr + 1) * GAMMA)."""
    with np.errstate(over="ignore"):
        ctr = np.asarray(ctr).astype(np.uint64)
        return mix64(np.uint64(key) + (ctr + _ONE) * GAMMA)


def make_key(seed, *streams):
    """Derive a stream key from a master seed and a tuple of small integers."""
    k = mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF))
    for s in streams:
        k = u64(k, np.uint64(int(s) & 0xFFFFFFFFFFFFFFFF))
    return np.uint64(k)


def u64_2(key, a, b):
    """Two-level counter: word b of the sub-stream a of `key` (a, b arrays broadcast)."""
    return u64(u64(key, a), b)


def uniform(words):
    """Map 64-bit words to doubles in [0, 1) using the top 53 bits."""
    return (np.asarray(words, dtype=np.uint64) >> _S11).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal(key, ctr):
    """Standard normal draws (float64) by the Box-Muller transform of two words."""
    ctr = np.asarray(ctr).astype(np.uint64)
    with np.errstate(over="ignore"):
        u1 = uniform(u64(key, ctr * np.uint64(2)))
        u2 = uniform(u64(key, ctr * np.uint64(2) + _ONE))
    # 1 - u1 lies in (0, 1], so the logarithm is finite
    return np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)
