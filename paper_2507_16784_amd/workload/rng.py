"""Counter-based integer PRNG for the synthetic workloads.

A splitmix64-style mixer over (seed, counter): every draw is a pure function of
the two integers, so a tree or a schedule regenerates identically anywhere.
Only integers come out of this module; no floating point is involved.
"""

_M64 = (1 << 64) - 1


def mix64(x: int) -> int:
    """Finalising mixer of splitmix64 (public-domain constants)."""
    x &= _M64
    x = (x + 0x9E3779B97F4A7C15) & _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


class Stream:
    """Sequential draws from one seed; draw i equals mix64(mix64(seed) + i)."""

    def __init__(self, seed: int):
        self._base = mix64(seed)
        self._i = 0

    def u64(self) -> int:
        v = mix64(self._base + self._i)
        self._i += 1
        return v

    def randint(self, lo: int, hi: int) -> int:
        """Uniform integer in [lo, hi] (inclusive); modulo bias is below 2**-40."""
        if hi < lo:
            raise ValueError("empty range")
        return lo + self.u64() % (hi - lo + 1)

    def permutation(self, n: int):
        """Fisher-Yates shuffle of range(n)."""
        p = list(range(n))
        for i in range(n - 1, 0, -1):
            j = self.u64() % (i + 1)
            p[i], p[j] = p[j], p[i]
        return p
