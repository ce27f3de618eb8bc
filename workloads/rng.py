"""Counter-based pseudo-random numbers for the synthetic workloads.

Every value is a pure function of (seed, index): value i of a stream is the
splitmix64 finaliser applied to seed + (i+1)*golden-gamma (Steele, Lea, Flood,
"Fast splittable pseudorandom number generators", OOPSLA 2014).  Normals come
from the Box-Muller transform of two consecutive uniforms.  Nothing here knows
anything about networks; callers pass shapes and counts.
"""
import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def u64(seed, start, count):
    """Values start..start+count-1 of the stream `seed` as uint64."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GAMMA)


def derive(seed, *tags):
    """A new 64-bit seed from a seed and integer tags (tensor index, query number ...)."""
    s = np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
    with np.errstate(over="ignore"):
        for t in tags:
            s = _mix(s + np.uint64((int(t) + 1) & 0xFFFFFFFFFFFFFFFF) * _GAMMA)
    return int(s)


def uniform(seed, start, count):
    """Doubles in [0,1) with 53 random bits."""
    return (u64(seed, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal(seed, count):
    """`count` standard normals (float64) from 2*ceil(count/2) uniforms."""
    half = (count + 1) // 2
    u = uniform(seed, 0, 2 * half)
    r = np.sqrt(-2.0 * np.log1p(-u[0::2]))
    th = (2.0 * np.pi) * u[1::2]
    out = np.empty(2 * half, dtype=np.float64)
    out[0::2] = r * np.cos(th)
    out[1::2] = r * np.sin(th)
    return out[:count]


class Stream:
    """Sequential view of one counter-based stream (for host-side sampling)."""

    def __init__(self, seed):
        self.seed = int(seed)
        self.pos = 0

    def next_u64(self):
        v = int(u64(self.seed, self.pos, 1)[0])
        self.pos += 1
        return v

    def next_uniform(self):
        v = float(uniform(self.seed, self.pos, 1)[0])
        self.pos += 1
        return v

    def randint(self, n):
        """Integer in [0, n)."""
        return int(self.next_uniform() * n) % n

    def permutation(self, n):
        """Fisher-Yates shuffle of range(n)."""
        p = list(range(n))
        for i in range(n - 1, 0, -1):
            j = self.randint(i + 1)
            p[i], p[j] = p[j], p[i]
        return p
