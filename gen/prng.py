"""Counter-based 64-bit generator used by every synthetic workload.

`bits(seed, stream, n)` is a pure function of its arguments: element `i` is the
SplitMix64 finaliser applied to `seed*K1 + stream*K2 + (i+1)*GOLDEN` (mod 2^64).
It depends on no library's distribution code, so the same workloads come out on
every machine and numpy version.  This module holds no arithmetic of the sparse
method itself; it only makes inputs.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_K1 = np.uint64(0xD1342543DE82EF95)
_K2 = np.uint64(0xA0761D6478BD642F)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def bits(seed, stream, n, offset=0):
    """`n` uint64 words of stream `stream` of generator `seed`, starting at counter `offset`."""
    with np.errstate(over="ignore"):
        base = np.uint64(seed) * _K1 + np.uint64(stream) * _K2
        ctr = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        return _mix(_mix(base) + ctr * _GOLDEN)


def uniform01(seed, stream, n, offset=0):
    """f64 in [0, 1) with 53 random bits."""
    return (bits(seed, stream, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform_pm1(seed, stream, n, dtype=np.float64):
    """i.i.d. U[-1, 1) in `dtype` (drawn in f64, rounded once)."""
    return (2.0 * uniform01(seed, stream, n) - 1.0).astype(dtype)


def small_ints(seed, stream, n, lo=-8, hi=8, dtype=np.float64):
    """Integers in [lo, hi] as floating point: products and sums of these are exact."""
    span = np.uint64(hi - lo + 1)
    return ((bits(seed, stream, n) >> np.uint64(16)) % span).astype(np.int64).astype(dtype) + dtype(lo)


def below(seed, stream, n, bound, offset=0):
    """Integers uniform in [0, bound) (bound < 2^53), int64."""
    return np.minimum((uniform01(seed, stream, n, offset) * float(bound)).astype(np.int64), bound - 1)


def normal(seed, stream, n):
    """Standard normals by the Box-Muller transform of two uniform streams."""
    u1 = 1.0 - uniform01(seed, stream, n)            # (0, 1]
    u2 = uniform01(seed, stream + 0x5EED, n)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def permutation(seed, stream, n):
    """A seeded permutation of range(n): the order of n random 64-bit keys (stable sort)."""
    return np.argsort(bits(seed, stream, n), kind="stable")
