"""Counter-based 64-bit generator, specified by its recurrence.

value(seed, stream, i) = mix64(seed * K1 + stream * K2 + (i + 1) * GOLDEN)   (mod 2^64)

mix64 is the splitmix64 finaliser (Steele, Lea, Flood 2014):
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27; z *= 0x94D049BB133111EB; z ^= z >> 31

Every draw is a pure function of (seed, stream, i), so arrays of any length can
be produced in vectorised form and reproduced element by element in pure Python
(tests do both and compare).
"""
import numpy as np

GOLDEN = 0x9E3779B97F4A7C15
K1 = 0xD1342543DE82EF95
K2 = 0xA0761D6478BD642F
M1 = 0xBF58476D1CE4E5B9
M2 = 0x94D049BB133111EB
MASK = (1 << 64) - 1


def mix64(z):
    """splitmix64 finaliser on numpy uint64 arrays (wrap-around arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = z ^ (z >> np.uint64(30))
        z = z * np.uint64(M1)
        z = z ^ (z >> np.uint64(27))
        z = z * np.uint64(M2)
        z = z ^ (z >> np.uint64(31))
    return z


def mix64_py(z):
    """Same finaliser on a Python int (used by tests as the second implementation)."""
    z &= MASK
    z ^= z >> 30
    z = (z * M1) & MASK
    z ^= z >> 27
    z = (z * M2) & MASK
    z ^= z >> 31
    return z


def raw_py(seed, stream, i):
    return mix64_py((seed * K1 + stream * K2 + (i + 1) * GOLDEN) & MASK)


class CounterRNG:
    """Stateless draws addressed by (stream, index)."""

    def __init__(self, seed):
        self.seed = int(seed)

    def raw(self, stream, n, offset=0):
        base = (self.seed * K1 + int(stream) * K2) & MASK
        idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        with np.errstate(over="ignore"):
            z = np.uint64(base) + idx * np.uint64(GOLDEN)
        return mix64(z)

    def uniform(self, stream, n, offset=0):
        """float64 in [0, 1): top 53 bits."""
        return (self.raw(stream, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))

    def normal(self, stream, n):
        """Standard normals by Box-Muller; draw 2k and 2k+1 feed normal k... pairs (2j, 2j+1)
        give normals 2j (cos branch) and 2j+1 (sin branch)."""
        npair = (n + 1) // 2
        u = self.uniform(stream, 2 * npair)
        u1 = 1.0 - u[0::2]            # (0, 1]
        u2 = u[1::2]
        r = np.sqrt(-2.0 * np.log(u1))
        out = np.empty(2 * npair, dtype=np.float64)
        out[0::2] = r * np.cos(2.0 * np.pi * u2)
        out[1::2] = r * np.sin(2.0 * np.pi * u2)
        return out[:n]

    def integers(self, stream, n, high):
        """Integers in [0, high) via the multiply-shift map floor(u * high) on the 53-bit uniform."""
        return np.minimum((self.uniform(stream, n) * high).astype(np.int64), high - 1)

    def permutation(self, stream, n):
        """Permutation of range(n): stable argsort of n raw 64-bit keys."""
        return np.argsort(self.raw(stream, n), kind="stable").astype(np.int64)
