"""Counter-based pseudo-random numbers for the synthetic workloads.

A self-contained SplitMix64 stream (Steele, Lea, Flood 2014) evaluated in closed
form: output i of stream `seed` is mix(seed + (i + 1) * GOLDEN). Being
counter-based, any slice of a stream can be produced on its own, by any thread,
and the draws do not depend on numpy's own generators or their versions.

Only random draws live here; nothing of the flow's arithmetic does.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK = (1 << 64) - 1


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _mix_int(z):
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def substream(seed, *ids):
    """Derive the seed of an independent stream from `seed` and integer ids."""
    s = _mix_int(int(seed) + 0x9E3779B97F4A7C15)
    for i in ids:
        s = _mix_int(s ^ _mix_int((int(i) + 1) * 0x9E3779B97F4A7C15))
    return s


def bits64(seed, n, offset=0):
    """Outputs offset .. offset+n-1 of stream `seed`, as uint64."""
    with np.errstate(over="ignore"):
        i = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        return _mix(np.uint64(seed & _MASK) + i * _GOLDEN)


def uniform01(seed, n, offset=0):
    """n doubles in [0, 1)."""
    return (bits64(seed, n, offset) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def randint(seed, n, lo, hi, offset=0):
    """n integers in [lo, hi) (multiply-shift on the top 32 bits)."""
    top = bits64(seed, n, offset) >> np.uint64(32)
    return (lo + ((top * np.uint64(hi - lo)) >> np.uint64(32)).astype(np.int64)).astype(np.int64)


def normal(seed, n):
    """n standard normals by Box-Muller; pair j yields cos and sin variates."""
    m = (n + 1) // 2
    b = bits64(seed, 2 * m)
    u1 = ((b[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)  # (0, 1]
    u2 = (b[1::2] >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)          # [0, 1)
    r = np.sqrt(-2.0 * np.log(u1))
    out = np.empty(2 * m, dtype=np.float64)
    out[0::2] = r * np.cos(2.0 * np.pi * u2)
    out[1::2] = r * np.sin(2.0 * np.pi * u2)
    return out[:n]


def shuffle(seed, n):
    """A permutation of 0..n-1: Fisher-Yates driven by the stream."""
    p = np.arange(n, dtype=np.int64)
    if n < 2:
        return p
    u = uniform01(seed, n - 1)
    for k in range(n - 1, 0, -1):
        j = int(u[n - 1 - k] * (k + 1))
        p[k], p[j] = p[j], p[k]
    return p
