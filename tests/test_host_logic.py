"""Host-side logic that needs no GPU: the index arithmetic the kernels rely on."""
import numpy as np


def _magic(d):
    return 0 if d <= 1 else (1 << 32) // d + 1


def _udiv_magic(u, d, m):
    """The kernels' division by a precomputed reciprocal, emulated with exact integers: high word of the
    32 x 32 product, then one multiply-and-compare."""
    if m == 0:
        return u
    q = (u * m) >> 32
    q &= 0xFFFFFFFF
    return q - 1 if ((q * d) & 0xFFFFFFFF) > u else q


def test_reciprocal_division_is_exact_over_the_admitted_range():
    """Sub-tile ids are below 2^30 / 16 and divisors (sub-tiles per image, per row) are arbitrary: the corrected
    form must be exact where the bare high-word estimate is not (power-of-two grids with many streams)."""
    rng = np.random.default_rng(5)
    bad_plain = 0
    for d in [2, 3, 4, 7, 16, 49, 64, 196, 4096, 16384, 65536, 12345, 99991, (1 << 20) + 3]:
        m = _magic(d)
        us = {0, 1, d - 1, d, d + 1, (1 << 26) - 1, (1 << 26), (1 << 30) - 1}
        us |= {k * d - 1 for k in (2, 1000, (1 << 26) // d) if k * d - 1 > 0}
        us |= {k * d for k in (2, 1000, (1 << 26) // d)}
        us |= set(int(v) for v in rng.integers(0, 1 << 30, size=2000))
        for u in us:
            assert _udiv_magic(u, d, m) == u // d, (u, d)
            bad_plain += ((u * m) >> 32) != u // d
    assert bad_plain > 0  # the uncorrected estimate does fail in this range: the correction is needed
    # the advisor's cases: last sub-tile of stream >= 16 at 32 streams of 128 x 128 sub-tiles
    d = 16384
    u = 17 * d - 1
    assert ((u * _magic(d)) >> 32) != u // d and _udiv_magic(u, d, _magic(d)) == u // d
