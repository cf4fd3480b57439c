"""Counter-based pseudo-random numbers for the synthetic workloads.

A value is a pure function of its key (seed, stream, counter): no state, so a
population can be regenerated piecewise, in any order, and identically on
every machine and numpy version.  The mixing function is the 64-bit finaliser
of SplitMix64 (Steele, Lea, Flood: "Fast splittable pseudorandom number
generators", OOPSLA 2014).
"""
import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)


def mix64(z):
    """SplitMix64 output function on a uint64 array (wrap-around arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def hash_u64(seed, stream, counter):
    """64 uniform bits for every element of `counter` under (seed, stream).

    `seed` and `stream` are Python ints (any size, reduced mod 2**64);
    `counter` is an integer array.
    """
    with np.errstate(over="ignore"):
        s = mix64(np.uint64(int(seed) & 0xFFFFFFFFFFFFFFFF) + _GOLDEN)
        s = mix64(s ^ (np.uint64(int(stream) & 0xFFFFFFFFFFFFFFFF) * _GOLDEN))
        c = np.asarray(counter).astype(np.uint64)
        return mix64(s + (c + np.uint64(1)) * _GOLDEN)


def uniform01(bits):
    """Map uint64 bits to float64 in [0, 1) using the top 53 bits."""
    return (np.asarray(bits, dtype=np.uint64) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
