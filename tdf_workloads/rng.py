"""SplitMix64 as a counter-based generator (Steele, Lea & Flood 2014; the public-domain
reference by Vigna): the i-th output is mix(seed + (i+1)*GAMMA), so any block of outputs
can be produced at once with NumPy's wrapping uint64 arithmetic.
"""
import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


class SplitMix64:
    """Stream of 64-bit words; `seed` and the running counter fully determine it."""

    def __init__(self, seed):
        self.seed = np.uint64(int(seed) & 0xFFFFFFFFFFFFFFFF)
        self.count = 0

    def u64(self, n):
        n = int(n)
        with np.errstate(over="ignore"):
            idx = np.arange(self.count + 1, self.count + n + 1, dtype=np.uint64)
            out = _mix(self.seed + idx * _GAMMA)
        self.count += n
        return out

    def fork(self, k):
        """Independent child stream number k (seeded by a word of a side stream)."""
        with np.errstate(over="ignore"):
            s = _mix((self.seed ^ np.uint64(0xD1B54A32D192ED03)) + np.uint64(int(k) + 1) * _GAMMA)
        return SplitMix64(int(s))

    def uniform(self, n):
        """n doubles in [0,1) from the top 53 bits of each word."""
        return (self.u64(n) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)

    def randint(self, lo, hi, n):
        """n integers uniform on the closed range [lo, hi]."""
        span = int(hi) - int(lo) + 1
        return (np.floor(self.uniform(n) * span).astype(np.int64) + int(lo)).clip(lo, hi)

    def normal(self, n):
        """n standard normals by Box-Muller (both branches used)."""
        m = (int(n) + 1) // 2
        u1 = 1.0 - self.uniform(m)          # (0,1]
        u2 = self.uniform(m)
        r = np.sqrt(-2.0 * np.log(u1))
        z = np.concatenate([r * np.cos(2.0 * np.pi * u2), r * np.sin(2.0 * np.pi * u2)])
        return z[: int(n)]

    def xavier_uniform(self, rows, cols):
        a = np.sqrt(6.0 / (rows + cols))
        return ((self.uniform(rows * cols) * 2.0 - 1.0) * a).reshape(rows, cols)
