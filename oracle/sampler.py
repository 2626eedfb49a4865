"""Per-iteration pattern sampling (test oracle, CPU only).

Section 3.4: each iteration draws a period dp from the distribution K, then a
bias b uniformly from {1..dp}.  The paper does not fix the random source; to
make masks reproducible bit for bit the draw is counter-based and integer only:
two 32-bit words from a stateless 64-bit mixer of (seed, iteration, stream id),
dp by inverse CDF on the 2^32 fixed-point table, b by multiply-shift.

The mixer is the public-domain SplitMix64 finaliser (Steele, Lea, Flood 2014;
constants 0xBF58476D1CE4E5B9 and 0x94D049BB133111EB, increment 0x9E3779B97F4A7C15).
"""
M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


def mix64(z: int) -> int:
    z &= M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def draw_words(seed: int, iteration: int, stream_id: int):
    """Two 32-bit words for (seed, iteration, stream)."""
    h = mix64((seed + GOLDEN) & M64)
    h = mix64((h ^ (iteration & M64)) + GOLDEN)
    h = mix64((h ^ (stream_id & 0xFFFFFFFF)) + GOLDEN)
    return h >> 32, h & 0xFFFFFFFF


def pattern_from_words(cdf, r1: int, r2: int):
    """(dp, b): dp = 1 + min{i : r1 < cdf[i]}, b = 1 + floor(r2 * dp / 2^32)."""
    dp = None
    for i, c in enumerate(cdf):
        if r1 < int(c):
            dp = i + 1
            break
    if dp is None:                       # cannot happen when cdf[-1] == 2^32
        dp = len(cdf)
    b = 1 + ((r2 * dp) >> 32)
    return dp, b


def sample_pattern(cdf, seed: int, iteration: int, stream_id: int):
    """Pattern of (seed, iteration, stream): first dp ~ K, then b ~ U{1..dp} (Section 3.4)."""
    r1, r2 = draw_words(seed, iteration, stream_id)
    return pattern_from_words(cdf, r1, r2)
