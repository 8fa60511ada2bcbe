"""The sampler skips the Gumbel variate of an entry whose score cannot win.  It decides that from
bounds on the variate that only look at the leading bit of the uniform's complement; a bound that
failed for some random word would silently drop a winner once in a long while, which random parity
runs need not catch.  Here the bounds are checked for every value the uniform can take (the variate
depends on the upper 23 bits of a random word), against the Gumbel transform in float64 and, on a
sample, against the oracle's binary32 routine."""
import numpy as np

import oracle

LN2 = np.log(2.0)


def _bounds(k):
    """k = the 23 bits of a random word that make the uniform u = (2 k + 1) 2^-24; returns c and the
    bounds (c - 1) ln2 <= G <= (c + 1) ln2 (lower bound -ln(24 ln 2) for c = 0), with the margins the
    kernel adds for the rounding of its logarithm routine."""
    m = (0x00FFFFFF ^ (k << 1)).astype(np.int64)            # (1 - u) 2^24: odd, 1 .. 2^24 - 1
    c = 23 - np.floor(np.log2(m.astype(np.float64))).astype(np.int64)   # clz of the 32-bit word minus 8
    upper = (c + 1) * 0.693148 + 1e-3
    lower = np.where(c >= 1, (c - 1) * 0.693147 - 1e-3 - 1e-6, -2.82)
    return m, c, lower, upper


def test_bounds_hold_for_every_uniform():
    k = np.arange(1 << 23, dtype=np.int64)
    m, c, lower, upper = _bounds(k)
    assert m.min() == 1 and m.max() == (1 << 24) - 1 and (m & 1).all()
    assert c.min() == 0 and c.max() == 23
    # the exponent really is the leading-zero count: 2^(23 - c) <= m < 2^(24 - c)
    assert ((m >> (23 - c)) == 1).all()
    u = (2 * k + 1).astype(np.float64) * 2.0 ** -24
    g = -np.log(-np.log(u))
    assert (g <= upper - 9e-4).all(), "upper bound"      # holds without the rounding margin
    assert (g >= lower + 9e-4).all(), "lower bound"
    # and they are not vacuous: two binades apart, as the kernel's comment says
    assert np.all(upper[c >= 1] - lower[c >= 1] < 2 * LN2 + 3e-3)


def test_bounds_hold_for_the_binary32_routine():
    oracle.build()
    rng = np.random.default_rng(11)
    ks = np.concatenate([rng.integers(0, 1 << 23, 20000), np.arange(0, 4096), (1 << 23) - 1 - np.arange(0, 4096),
                         (1 << np.arange(0, 23)), (1 << np.arange(1, 23)) - 1]).astype(np.int64)
    _, _, lower, upper = _bounds(ks)
    low_bits = rng.integers(0, 512, ks.size)
    for k, lb, lo, up in zip(ks, low_bits, lower, upper):
        g = oracle.gumbel(int((k << 9) | lb))   # the lower 9 bits of the word do not matter
        assert lo <= g <= up, (k, g, lo, up)
