"""Counter-based 64-bit generator used for every random draw of the subnet generator.

Test infrastructure (see the package docstring).  The paper only says that seeds are
fixed (Section 4, "Hardware Setup"); it names no generator, so this build fixes one:

  mix(z):   z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27;
            z *= 0x94D049BB133111EB; z ^= z >> 31            (all mod 2^64)
  stream key for (seed, round, layer, kind):
            x = mix(seed); x = mix(x + round); x = mix(x + layer); x = mix(x + kind)
  draw:     x += 0x9E3779B97F4A7C15; return mix(x)            (SplitMix64's step)
  below(n): draw until the 64-bit value v < 2^64 - (2^64 mod n); return v mod n
            (rejection, so the result is exactly uniform and no floating point is used)
"""
MASK = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


def mix(z: int) -> int:
    z &= MASK
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & MASK
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & MASK
    z ^= z >> 31
    return z


class Stream:
    """One independent stream per (seed, round, layer, kind)."""

    def __init__(self, seed: int, rnd: int = 0, layer: int = 0, kind: int = 0, *, raw_state=None):
        if raw_state is not None:
            self.x = raw_state & MASK
            return
        x = mix(seed)
        x = mix(x + rnd)
        x = mix(x + layer)
        x = mix(x + kind)
        self.x = x

    def u64(self) -> int:
        self.x = (self.x + GOLDEN) & MASK
        return mix(self.x)

    def below(self, n: int) -> int:
        """Uniform integer in [0, n)."""
        assert n >= 1
        limit = (1 << 64) - ((1 << 64) % n)
        while True:
            v = self.u64()
            if v < limit:
                return v % n

    def shuffle(self, a: list) -> None:
        """Fisher-Yates, i descending from len-1 to 1, swap with uniform j in [0, i]."""
        for i in range(len(a) - 1, 0, -1):
            j = self.below(i + 1)
            a[i], a[j] = a[j], a[i]

    def unique_choice(self, pool: list, m: int) -> list:
        """m distinct elements of `pool`, uniform without replacement: the first m slots of a
        partial Fisher-Yates that walks t = 0..m-1 and swaps slot t with a uniform slot in [t, len)."""
        a = list(pool)
        for t in range(m):
            j = t + self.below(len(a) - t)
            a[t], a[j] = a[j], a[t]
        return a[:m]
